// Test hooks (include/harli_debug.h): single kernels exposed for the GPU tests.
#include "harli_debug.h"

#include "ctx.h"
#include "gemm.h"

using namespace harli;

extern "C" harli_status harli_dbg_gemm(const void* A1, const void* B1, int32_t K1, const void* A2, const void* B2, int32_t K2,
                                       int32_t M, int32_t N, float alpha, int32_t causal, int32_t half, void* Cb,
                                       float* Cf, const float* res, void* Ct, void* hip_stream) {
  GemmArgs g{};
  g.M = M;
  g.N = N;
  g.nb1 = g.nb2 = 1;
  g.alpha = alpha;
  g.causal = causal;
  g.half = half;
  g.nseg = 0;
  auto seg = [&](const void* A, const void* B, int K) {
    GemmSeg& s = g.seg[g.nseg++];
    s = GemmSeg{};
    s.A = static_cast<const unsigned short*>(A);
    s.B = static_cast<const unsigned short*>(B);
    s.K = K;
    s.lda = s.ldb = K;
  };
  seg(A1, B1, K1);
  if (K2 > 0) seg(A2, B2, K2);
  g.Cb = static_cast<unsigned short*>(Cb);
  g.ldcb = N;
  g.Cf = Cf;
  g.res = res;
  g.ldcf = N;
  g.Ct = static_cast<unsigned short*>(Ct);
  g.ldct = M;
  return gemm_launch(g, 1, static_cast<hipStream_t>(hip_stream));
}

extern "C" harli_status harli_prof_enable(int32_t on) {
  gemm_prof_enable(on != 0);
  return HARLI_OK;
}

extern "C" harli_status harli_prof_collect(double* gemm_flops, double* gemm_ms, int64_t* gemm_launches) {
  if (!gemm_flops || !gemm_ms || !gemm_launches) return fail(HARLI_ERR_INVALID, "prof_collect: null argument");
  long long n = 0;
  harli_status s = gemm_prof_collect(gemm_flops, gemm_ms, &n);
  *gemm_launches = n;
  return s;
}
