// Adapter update: AdamW with decoupled weight decay (Harli Sec. 2.1 names forward, backward, update; the optimizer
// itself is this build's reading).  One element per thread, fp32 arithmetic, fp32 master parameters with a bf16 copy
// for the kernels that read the adapters.
#include <cmath>

#include "ctx.h"
#include "device_utils.h"

namespace harli {
namespace {
__global__ void __launch_bounds__(256) k_adamw(float* __restrict__ master, float* __restrict__ m, float* __restrict__ v,
                                               float* __restrict__ grad, unsigned short* __restrict__ param, size_t n, float lr,
                                               float b1, float b2, float eps, float wd, float gscale, float inv_c1, float inv_c2,
                                               int zero_grad) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float g = grad[i] * gscale;
  const float mi = b1 * m[i] + (1.f - b1) * g;
  const float vi = b2 * v[i] + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  float p = master[i];
  p -= lr * ((mi * inv_c1) / (sqrtf(vi * inv_c2) + eps) + wd * p);
  master[i] = p;
  if (param) param[i] = f2bf(p);
  if (zero_grad) grad[i] = 0.f;
}
}  // namespace
}  // namespace harli

extern "C" harli_status harli_adamw_step(float* master, float* m, float* v, float* grad, void* param_bf16, size_t n,
                                         const harli_adamw_cfg* cfg, void* hip_stream) {
  using namespace harli;
  if (!master || !m || !v || !grad || !cfg) return fail(HARLI_ERR_INVALID, "adamw_step: null argument");
  if (cfg->step < 1 || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
    return fail(HARLI_ERR_INVALID, "adamw_step: step %d, betas %g %g", cfg->step, cfg->beta1, cfg->beta2);
  if (n == 0) return HARLI_OK;
  // bias corrections in double on the host
  const double c1 = 1.0 - std::pow((double)cfg->beta1, (double)cfg->step), c2 = 1.0 - std::pow((double)cfg->beta2, (double)cfg->step);
  hipLaunchKernelGGL(k_adamw, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), master, m, v,
                     grad, static_cast<unsigned short*>(param_bf16), n, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps,
                     cfg->weight_decay, cfg->grad_scale, (float)(1.0 / c1), (float)(1.0 / c2), cfg->zero_grad);
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}
