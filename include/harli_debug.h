/*
 * harli_debug.h -- test hooks of libharli.  NOT part of the stable ABI: they expose single
 * kernels so that the GPU tests can check them in isolation.
 */
#ifndef HARLI_DEBUG_H
#define HARLI_DEBUG_H

#include "harli.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The weight GEMM of the finetune unit (256-wide tiles, weight side in blocked order) on its own.  The descriptor
 * mirrors the kernel's arguments; weight-side operands are given ROW-MAJOR here ([rows, K], the contraction index
 * contiguous, 16-bit elements of the type `half` selects) and the hook makes their blocked copies itself (it allocates
 * device memory for them, synchronises the stream and frees them before it returns).
 *   C = alpha * sum_s A_s . B_s^T (+ res).  Segment s contributes to the output column tiles [tile0, tile1) (256
 *   columns per tile; 128 + 128 interleaved in 32-column groups when `pair` is set: B_s and B2_s are then the two
 *   matrices of the pair and either may be NULL) and its weight rows start at the first column of tile0.  Output block
 *   o starts at tile out_tile0[o] and has out_n[o] valid columns; all blocks are 16-bit (cb) or all fp32 (cf, optional
 *   res).  epi 0: plain; 2: SwiGLU backward (cf/cb unused: o0 = da, o1 = du from e0 = a, e1 = u); 3: gate/up pair
 *   (cb[0] = a, o1 = u, o0 = silu(a) * u).  tile_rows 128 or 256 fixes the tile height, 0 leaves the choice to the
 *   library.  reps > 1 repeats the launch and writes TFLOP/s over HIP events and the shader clock of the last launch
 *   to the host pointers (either may be NULL). */
typedef struct {
  int32_t M, nseg, nout, tiles_n, half, epi, tile_rows, reps;
  float alpha;
  const void* A[12];
  int64_t lda[12];
  int32_t K[12];
  const void* B[12];
  int32_t b_rows[12];
  const void* B2[12];
  int32_t b2_rows[12];
  int32_t tile0[12], tile1[12], pair[12];
  int32_t out_tile0[3], out_n[3];
  void* cb[3];
  int64_t ldcb[3];
  float* cf[3];
  const float* res[3];
  int64_t ldcf[3];
  const void *e0, *e1;
  void *o0, *o1;
  int64_t lde;
  int32_t* overflow_flag;
  double* tflops;
  double* shader_mhz;
  /* Compute units the tile height is chosen for: 0 = those of `hip_stream` (all of the device unless it is a
   * harli_cu_stream), n > 0 = n. */
  int32_t n_cu;
} harli_dbg_gemm2_desc;
harli_status harli_dbg_gemm2(const harli_dbg_gemm2_desc* d, void* hip_stream);

/* The grid the weight GEMM would launch for M rows and tiles_n column tiles at tile height tile_rows (128 or 256), and
 * its cost on n_cu compute units (host logic only, no device needed).  out[6] (host) receives GM, GN, total, chunk,
 * grid and the rounds of tiles over the compute units.  Workgroup w computes the tile in slot (w % 8) * chunk + w / 8
 * of the XCD-aware order: blocks of GM x GN tiles, row-major inside a block and over the blocks; slots past the matrix
 * are idle.  The library launches the tile height with the smaller cost, a round of 128-row tiles counted as 0.55 of a
 * round of 256-row tiles. */
harli_status harli_dbg_gemm2_plan(int32_t M, int32_t tiles_n, int32_t tile_rows, int32_t n_cu, int32_t* out);

/* How one GEMM of a decode step above 32 sequences is cut (host logic only, no device needed): `batch` sequences,
 * n_mat (1, or 2 for gate and up) weight matrices of n_rows rows, contraction length K, on n_cu compute units, with
 * ws_bytes of workspace for the partial tiles.  out[7] (host): batch rows per tile / 64, batch tiles, rows of a partial
 * matrix, 256-row weight tiles of all matrices, ranges of K (0: not even one fits the workspace), rounds of workgroups
 * over the compute units, bytes of workspace used. */
harli_status harli_dbg_decode_gemm_plan(int32_t batch, int32_t n_rows, int32_t n_mat, int32_t K, int32_t n_cu, int64_t ws_bytes,
                                        int64_t* out);

/* Times one such GEMM on operands the call allocates, fills and frees (device memory; not for a caller that may not
 * allocate): the partial products, then their sum with the residual epilogue (n_mat 1) or the SwiGLU epilogue
 * (n_mat 2).  ksplit > 0 fixes the ranges of K, 0 leaves the choice to the plan.  out_us[4] (host): average microseconds
 * of the first and of the second launch over `reps` runs, the ranges of K and the tile height / 64 that ran. */
harli_status harli_dbg_decode_gemm_time(int32_t batch, int32_t n_rows, int32_t n_mat, int32_t K, int32_t ksplit, int32_t reps,
                                        float* out_us, void* hip_stream);

/* Measurement hook: the smallest batch whose decode steps run the tiled GEMMs (process-wide; 0 gives the library's
 * own threshold back).  A context takes the workspace of that path when its max_batch is 17 or more. */
void harli_dbg_decode_large_min_batch(int32_t batch);

/* The residency plan of harli_ft_window_* on its own (host logic only, no device needed): a window of n_slots over the
 * 2 * n_layers cyclic items, prefilled with items 0..n_slots-1, is driven through `items[0..n_access)`; for every
 * access the slot that served it, the item loaded on demand (-1 on a hit) and the item loaded into the slot
 * afterwards (-1 = none) are written to the three host arrays. */
harli_status harli_dbg_window_plan(int32_t n_layers, int32_t n_slots, const int32_t* items, int32_t n_access, int32_t* slot,
                                   int32_t* miss, int32_t* refill);

/* Kernel timing for the benchmark.  harli_prof_enable(n), n > 0: from now on every n-th launch of the
 * finetune unit's MFMA GEMM (the first, the (n+1)-th, ...) is bracketed by two HIP events on the stream it is
 * launched on; n <= 0 switches it off.  (An event pair costs the stream about 10 us of overlap between
 * neighbouring kernels: timing every launch slows a finetune unit by more than a tenth, so a benchmark samples.)
 * harli_prof_collect waits for the recorded events (it SYNCHRONISES on them), returns the summed algorithmic
 * flops (2*M*N*K per launch, half of that for causal launches) and the summed event-to-event milliseconds of the
 * timed launches and their number (all host pointers), and clears the record.  Not thread-safe. */
harli_status harli_prof_enable(int32_t on);
harli_status harli_prof_collect(double* gemm_flops, double* gemm_ms, int64_t* gemm_launches);

/* Measured memory ceilings of this GPU, for reading the roofline fractions.  Runs a plain read kernel on
 * `buf` (device, `bytes` long, contents irrelevant, at least 64 MiB) and writes the achieved GB/s to *gbs
 * (host).  mode 0: every workgroup streams a region of its own once per pass (HBM rate; use a buffer much
 * larger than the 256 MiB memory-side cache).  mode 1: workgroups re-read 32 shared 3 MiB regions the way the
 * MFMA GEMM's workgroups re-read operand panels (the rate at which the per-XCD L2 caches feed the CUs).
 * Synchronises the stream.  Returns HARLI_ERR_INVALID for a null pointer, a small buffer or an unknown mode. */
harli_status harli_dbg_read_bandwidth(const void* buf, size_t bytes, int32_t mode, double* gbs, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HARLI_DEBUG_H */
