// Weight GEMM of the finetune unit for gfx950:  C = alpha * sum_s A_s . B_s^T  (+ res), 16-bit operands, fp32 accumulate
// (Harli Sec. 2.1: PEFT is dominated by products with the frozen base weights; the LoRA path and frozen biases ride as
// further K segments).
//
// A_s is an activation [M, K_s], row-major with row stride lda.  B_s is a weight-side operand [N, K_s] kept in the
// BLOCKED layout this kernel streams: [row tile of 256][k step of 32][256 rows][32 k], rows past N and k past K_s
// zero.  A stage of a tile (256 rows x 32 k = 16 KiB) is contiguous in memory, so every wavefront load of it is one
// 1 KiB burst; measured on this chip a workgroup pulls such tiles at 41 B/clk/CU against 22 B/clk/CU for the same
// bytes gathered from row-major rows 8 KiB apart.  The library owns every weight-side operand (private copies of the
// frozen weights, per-call copies of the adapters), so it is free to keep them in this order.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"
#include "gemm_timer.h"

namespace harli {

constexpr int kG2TileN = 256, kG2StepK = 32;
constexpr int kGemm2MaxSeg = 12, kGemm2MaxOut = 3;

// elements of a blocked operand with N rows and contraction length K
__host__ __device__ inline size_t blocked_elems(long long N, long long K) {
  return (size_t)((N + kG2TileN - 1) / kG2TileN) * (size_t)((K + kG2StepK - 1) / kG2StepK) * (kG2TileN * kG2StepK);
}

// bytes of one finetune-private copy of a frozen [out, in] weight: the forward operand [out rows, in] and the backward
// operand [in rows, out] are padded differently, the copies are allocated (and moved by the weight window) at the larger
inline size_t ft_weight_copy_bytes(int out, int in) { return 2 * (blocked_elems(out, in) > blocked_elems(in, out) ? blocked_elems(out, in) : blocked_elems(in, out)); }

struct Gemm2Seg {
  const unsigned short* A;  // [M, K], row stride lda (multiple of 8), 16-byte aligned
  long long lda;
  int K;                    // multiple of 8
  const unsigned short* B;  // blocked [tile1 - tile0 row tiles][ceil(K/32)][256][32]
  // this segment contributes to the output column tiles [tile0, tile1) only (a fused launch stacks several weight
  // matrices along N, each with its own operand); B's first row tile is output tile tile0
  int tile0, tile1;
  // Interleaved pair (the gate and up projections in one launch): when B2 is set, the 256 columns of output tile t
  // are 128 columns of B and the same 128 columns of B2, alternating in groups of 32: tile column 64 g + c comes
  // from B row 128 (t - tile0) + 32 g + c for c < 32 and from B2 row 128 (t - tile0) + 32 g + c - 32 for c >= 32.
  // Either of B, B2 may then be null (that half contributes zeros: an adapter of one projection only).
  const unsigned short* B2;
  int pair;  // 0: plain, 1: interleaved pair
  // rows the blocked copies were made for (B and B2 alike): gemm2_launch checks that the tile range stays inside them
  int rows;
};

// One block of output columns: tiles [tile0, tile0 of the next block) hold columns 0.. of this block's matrices.
struct Gemm2Out {
  int tile0;
  int N;  // valid columns of this block
  unsigned short* Cb;  // 16-bit row-major or null
  long long ldcb;
  float* Cf;           // fp32 row-major or null
  const float* res;    // added to Cf (same layout) or null
  long long ldcf;
};

enum Gemm2Epi {
  GEMM2_EPI_NONE = 0,        // plain outputs (the kernel variant for fp32 outputs is picked from out[0].Cf)
  GEMM2_EPI_F32 = 1,         // internal: the variant that writes fp32 (+ residual, + optional 16-bit copy)
  GEMM2_EPI_SWIGLU_BWD = 2,  // as GEMM_EPI_SWIGLU_BWD: C = dm, o0 = da, o1 = du from e0 = a, e1 = u (row stride lde)
  GEMM2_EPI_GATEUP = 3       // interleaved pair: a = gate, u = up (16-bit), and o0 = m = silu(a) * u; out[0].Cb = a, o1 = u
};

struct Gemm2Args {
  int M, nseg, nout;
  Gemm2Seg seg[kGemm2MaxSeg];
  Gemm2Out out[kGemm2MaxOut];
  int tiles_n;  // output column tiles in all blocks together
  float alpha;
  int half;     // operands and 16-bit outputs are IEEE half (1) or bfloat16 (0)
  int epi;
  const unsigned short *e0, *e1;
  unsigned short *o0, *o1;
  long long lde;
  int* overflow_flag;  // device int: bit 8 is set when a 16-bit output had to be clamped to the element's range (or null)
  long long* clk;      // clock probe (or null): workgroup 0 writes {shader-clock cycles, 100 MHz ticks} of its K loop
  // compute units the launch's stream may use (Harli Sec. 6.2: the finetune task runs on a share of them); 0: taken
  // from the stream (harli_cu_stream_create), else the whole device.  The tile height is chosen for it.
  int n_cu;
};


harli_status gemm2_launch(const Gemm2Args& a, hipStream_t st);

// The grid gemm2_launch would use (exposed for the host-side tests of the tile order).
struct Gemm2Plan {
  int GM, GN, total, chunk, grid;  // block of tiles per XCD pass, padded tile slots, slots per XCD, workgroups launched
  int rounds;                      // rounds of tiles over the compute units
};
Gemm2Plan gemm2_plan(int M, int tiles_n, int FM, int n_cu);

// Blocked copies.  src is [R][C] row-major in the storage type (bf16; fp32 when src_f32 is 1; 16-bit elements that
// are already in the compute element and are copied bit for bit when src_f32 is 2); the operand is B[n][k] =
// src[n][k] (transpose 0: N = R, K = C) or src[k][n] (transpose 1: N = C, K = R).  dst must hold blocked_elems(N, K)
// elements; every element of it is written (zeros in the padding).
struct BlockJob {
  const void* src;
  unsigned short* dst;
  int R, C, transpose, src_f32;
};
struct BlockJobs {
  BlockJob j[16];
  int n;
  int half;   // destination element: IEEE half (1) or bfloat16 (0)
  int* flag;  // device int or null: bit 8 is set when a converted value lay beyond the destination element's range
};
void gemm2_block_jobs(const BlockJobs& jobs, hipStream_t st);
// measurement hook: 128 or 256 fixes the tile height of every later launch, anything else gives the choice back
void gemm2_force_tile_rows(int rows);
// compute units a stream made by harli_cu_stream_create may use; 0 for any other stream (sched.cpp)
int cu_stream_count(void* hip_stream);

}  // namespace harli
