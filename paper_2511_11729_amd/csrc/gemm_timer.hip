// Per-launch timing of the finetune unit's GEMMs for the benchmark (harli_prof_*).
#include "gemm_timer.h"

#include "ctx.h"

#include <vector>

namespace harli {

// ---- optional per-launch timing (harli_prof_*): two events around every n-th GEMM launch ----
namespace {
struct ProfRec {
  hipEvent_t e0, e1;
  double flops;
};
int g_prof_every = 0;       // 0: off; n: the launches whose running number is a multiple of n are timed
long long g_prof_seen = 0;  // launches since enabling
std::vector<ProfRec> g_prof;
}  // namespace

void gemm_prof_enable(int every) {
  g_prof_every = every > 0 ? every : 0;
  g_prof_seen = 0;
}

harli_status gemm_prof_collect(double* flops, double* ms, long long* launches) {
  double f = 0.0, t = 0.0;
  for (ProfRec& r : g_prof) {
    HARLI_HIP(hipEventSynchronize(r.e1));
    float dt = 0.f;
    HARLI_HIP(hipEventElapsedTime(&dt, r.e0, r.e1));
    f += r.flops;
    t += dt;
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  *flops = f;
  *ms = t;
  *launches = (long long)g_prof.size();
  g_prof.clear();
  return HARLI_OK;
}

hipError_t GemmTimer::begin(double flops_of_launch, hipStream_t st) {
  if (!(g_prof_every > 0 && (g_prof_seen++ % g_prof_every) == 0)) return hipSuccess;
  hipEvent_t a, b;
  hipError_t e = hipEventCreate(&a);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&b);
  if (e != hipSuccess) return e;
  e0 = a, e1 = b, flops = flops_of_launch;
  return hipEventRecord(a, st);
}
hipError_t GemmTimer::end(hipStream_t st) {
  if (!e0) return hipSuccess;
  hipError_t e = hipEventRecord(static_cast<hipEvent_t>(e1), st);
  g_prof.push_back(ProfRec{static_cast<hipEvent_t>(e0), static_cast<hipEvent_t>(e1), flops});
  e0 = e1 = nullptr;
  return e;
}

}  // namespace harli
