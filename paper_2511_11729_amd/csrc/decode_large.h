// Decode step, shared between the small-batch kernels (decode.hip) and the large-batch path (decode_large.hip).
//
// Large batches (Harli Sec. 1: a decode instance is served at batch sizes up to 256 before it saturates): above 32
// sequences the step's GEMMs are no longer pure weight streams -- every 16-row weight tile would be multiplied with
// 4..16 batch fragments that each wave pulls through the vector cache for itself.  The large-batch path runs them as
// tiled MFMA GEMMs instead: both operands staged through LDS once per workgroup, the contraction cut into ranges over
// workgroups so that the few output tiles of a narrow projection still fill the chip, fp32 partial tiles written to a
// workspace, and a second small kernel per GEMM that adds the partials in a fixed order and applies the step's
// epilogue (norm factor, biases, rotary embedding, KV append; residual and next operand; SwiGLU).
#pragma once
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace harli {

// Element (jb, k) of an x operand with `steps` = ceil(K/32) k-steps, fragment order:
// [batch tile][k-step][lane = (k%32)/8*16 + jb%16][8].
__device__ __forceinline__ size_t xfrag_off(int jb, int k, int steps) {
  return ((((size_t)(jb >> 4) * steps + (k >> 5)) * 64) + ((k >> 3) & 3) * 16 + (jb & 15)) * 8 + (k & 7);
}

struct SkinnyArgs {
  const unsigned short* x;  // fragment-order operand
  int B, b0, K;             // batch size, first batch row of this pass, contraction length
  int n_rows;               // output rows (tail masking of stores)
  const unsigned short *w0, *w1;  // pre-shuffled weights
  const float* ssq_in;  // partial sums of squares of the operand's source row (rho): [row][ssq_np], or null
  int ssq_np;           // entries per row (a multiple of 16; entries past the producer's tiles are zero)
  float eps, inv_dim;
  // QKV
  float* qbuf;
  const float* rope;
  const int* kv_len;
  const int* page_table;
  int max_pages, layer, n_q, n_kv, d;
  char* slab;
  KvGeom geom;
  int* err_flag;
  const float* bias[3];  // q, k, v biases (fp32, indexed by output row of that projection) or null
  // RESID
  const float* res;
  float* out;
  const float* gnext;
  unsigned short* hxn;  // next operand (fragment order, K = n_rows) or null
  float* ssq_out;       // [row][ssq_np]: this launch writes entry `tile` of every row it finishes
  // GATEUP
  unsigned short* mbuf;  // next operand (fragment order, K = n_rows)
  // LM
  float* logits;
};

// Sum of squares of a residual row (the next RMSNorm's denominator).  The row is produced 16 columns per weight tile
// by many workgroups, which finish in any order, and a float sum taken in completion order differs in its last bit
// from run to run (which then flips bf16 roundings downstream).  So nothing is accumulated across workgroups: every
// tile writes its own partial to entry `tile` of the row, and the kernel that needs the sum adds the row's entries in
// a fixed order (lane group g takes the float4 chunks g, g + 4, ..; then the four groups are added).  No atomics,
// and the bits of a step do not depend on scheduling.
__device__ __forceinline__ float ssq_row_sum(const float* row, int np, int g) {
  float s = 0.f;
  for (int i = g * 4; i < np; i += 16) {
    const float4 v = *reinterpret_cast<const float4*>(row + i);
    s += (v.x + v.y) + (v.z + v.w);
  }
  s += __shfl_xor(s, 16, 64);
  s += __shfl_xor(s, 32, 64);
  return s;
}


// ---- large-batch path ---------------------------------------------------------------------------------------------
enum DgKind { DG_QKV = 0, DG_RESID = 1, DG_GATEUP = 2, DG_LM = 3 };

// How one GEMM of the step is cut: (64 FM)-row batch tiles x 256-row weight tiles x ksplit ranges of K.
struct DgPlan {
  int FM, tiles_m, Mpad;  // batch rows per tile / 64, batch tiles, rows of a partial matrix (tiles_m * 64 FM)
  int tiles_n;            // 256-row weight tiles of all matrices of the launch together
  int ksplit;             // ranges of K; every range is a workgroup of its own per output tile
  int rounds;             // rounds of workgroups over the compute units
  size_t part_bytes;      // workspace the partial tiles need: ksplit * Mpad * tiles_n * 256 floats
};
// n_rows: output rows of one weight matrix; n_mat: matrices in the launch (2 for gate and up, else 1).  ws_bytes caps
// the workspace (ksplit falls until the partials fit).
DgPlan dg_plan(int B, int n_rows, int n_mat, int K, int n_cu, size_t ws_bytes);
// workspace a context needs for batches up to max_batch (0 when the large-batch path can never run)
size_t dg_workspace_bytes(const harli_model_cfg& m, int n_cu);
// once per process, before the first launch (harli_ctx_create calls it when it takes the workspace)
harli_status dg_init();
// One GEMM of the step with its epilogue; `a` as the small-batch kernels take it (b0 ignored: all rows at once).
// x_tiles: 16-row batch tiles the operand buffer was allocated for.  part: workspace of part_bytes.
harli_status dg_launch(DgKind kind, const SkinnyArgs& a, int x_tiles, float* part, size_t part_bytes, int n_cu, hipStream_t st);
// its two launches on their own (the partial products; their sum with the epilogue), and a measurement hook that fixes
// the number of K ranges of every later plan (0 gives the choice back)
harli_status dg_gemm(DgKind kind, const SkinnyArgs& a, int x_tiles, float* part, size_t part_bytes, int n_cu, hipStream_t st, DgPlan* used);
harli_status dg_epilogue(DgKind kind, const SkinnyArgs& a, const DgPlan& p, const float* part, hipStream_t st);
void dg_force_ksplit(int ksplit);
// smallest batch that takes the tiled path (measurement hook; 0 gives the default back)
void dg_set_min_batch(int b);
int dg_min_batch();

}  // namespace harli
