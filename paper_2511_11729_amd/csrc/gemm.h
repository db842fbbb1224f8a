// 16-bit MFMA GEMM used by the finetune unit:  C[z] = alpha * sum_s A_s[z] . B_s[z]^T  (+ res)
// Every operand is "NT": A_s is [M, K_s] and B_s is [N, K_s], both row-major with the
// contraction index contiguous.  Up to six K segments accumulate into one output, which is
// how the LoRA path rides on the base GEMM (y = [x | s*xA] . [W | B^T]^T, Sec. 2.1 LoRA) and
// how gradients that sum over several projections are formed in one pass.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace harli {

constexpr int kGemmMaxSeg = 6;

struct GemmSeg {
  const unsigned short* A;  // bf16 [M, K], row stride lda
  const unsigned short* B;  // bf16 [N, K], row stride ldb
  int K;                    // multiple of 8
  long long lda, ldb;
  // batch strides (elements); z -> (z0, z1, z2) = (z / (nb1*nb2), (z / nb2) % nb1, z % nb2)
  long long a_bs0, a_bs1, a_bs2, b_bs0, b_bs1, b_bs2;
};

enum GemmCausal {
  GEMM_FULL = 0,
  GEMM_OUT_LOWER = 1,  // only tiles touching n <= m are computed (rows = queries, cols = keys)
  GEMM_OUT_UPPER = 2,  // only tiles touching n >= m are computed (rows = keys, cols = queries)
  GEMM_K_UPTO_M = 3,   // A[m, k] is zero for k > m: the K loop stops at the tile's last row
  GEMM_K_FROM_M = 4    // A[m, k] is zero for k < m: the K loop starts at the tile's first row
};

struct GemmArgs {
  int M, N, nseg, nb1, nb2;  // nb1, nb2 >= 1; grid.z = number of batches
  GemmSeg seg[kGemmMaxSeg];
  float alpha;
  int causal;
  int half;  // operands and 16-bit outputs are IEEE half (1) or bfloat16 (0)
  // outputs (any subset): bf16 row-major, fp32 row-major (optionally + res), bf16 transposed [N, M]
  unsigned short* Cb;
  long long ldcb, cb_bs0, cb_bs1, cb_bs2;
  float* Cf;
  const float* res;  // same layout as Cf
  long long ldcf, cf_bs0, cf_bs1, cf_bs2;
  unsigned short* Ct;
  long long ldct, ct_bs0, ct_bs1, ct_bs2;
  // fused SwiGLU epilogues (not batched; N and lde multiples of 8, 16-byte aligned pointers, row stride lde):
  //   GEMM_EPI_SILU_MUL   C = the up projection u:  Cb = u (16-bit), o0 = silu(e0) * u   with e0 = the gate output a
  //   GEMM_EPI_SWIGLU_BWD C = dm:  o0 = da = dm * u * sig(a) * (1 + a (1 - sig(a))),  o1 = du = dm * a * sig(a),
  //                       e0 = a, e1 = u; no other output is written
  int epi;
  const unsigned short *e0, *e1;
  unsigned short *o0, *o1;
  long long lde;
  // Clock probe (null: off).  Workgroup 0 writes {shader-clock cycles, ticks of the constant 100 MHz counter} spent in
  // its K loop, so that the host can see at which clock the chip ran the launch.
  long long* clk;
};
enum GemmEpi { GEMM_EPI_NONE = 0, GEMM_EPI_SILU_MUL = 1, GEMM_EPI_SWIGLU_BWD = 2 };

// Launches on `st`; batches = grid.z.  Shapes are validated (K % 8, pointers, strides % 8).
harli_status gemm_launch(const GemmArgs& a, int batches, hipStream_t st);

// Per-launch timing for the benchmark: when enabled every gemm_launch is bracketed by two events on
// its stream; collect() waits for them and returns the summed flops, milliseconds and launch count.
void gemm_prof_enable(int every);
// The same bracket for other GEMM kernels: begin() before the launch, end() after it; both do nothing for launches
// that are not sampled.
struct GemmTimer {
  void *e0 = nullptr, *e1 = nullptr;
  double flops = 0;
  hipError_t begin(double flops_of_launch, hipStream_t st);
  hipError_t end(hipStream_t st);
};
harli_status gemm_prof_collect(double* flops, double* ms, long long* launches);

}  // namespace harli
