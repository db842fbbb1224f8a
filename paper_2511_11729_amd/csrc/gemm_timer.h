// Per-launch timing of GEMM kernels for the benchmark: when enabled, every n-th launch is bracketed by two events on
// its stream; collect() waits for them and returns the summed flops, milliseconds and launch count.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace harli {

void gemm_prof_enable(int every);
// begin() before the launch, end() after it; both do nothing for launches that are not sampled
struct GemmTimer {
  void *e0 = nullptr, *e1 = nullptr;
  double flops = 0;
  hipError_t begin(double flops_of_launch, hipStream_t st);
  hipError_t end(hipStream_t st);
};
harli_status gemm_prof_collect(double* flops, double* ms, long long* launches);

}  // namespace harli
