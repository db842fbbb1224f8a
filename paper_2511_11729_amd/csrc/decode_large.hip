// Large-batch GEMMs of the decode step (see decode_large.h): partial products on 32x32x16 bf16 MFMA tiles, then one
// small kernel per GEMM that adds the partials and applies the step's epilogue.
//
// k_dgemm<FM>: workgroup tile (64 FM) batch rows (FM = 1..4) x 256 weight rows over a range of K; four waves, one per
// SIMD, each a (32 FM) x 128 block.  Both operands are read where the small-batch kernels keep them -- MFMA-fragment
// order, [16-row tile][k step of 32][lane][8], a 16 x 32 tile being 1 KiB contiguous -- and go straight into LDS with
// buffer loads, tile by tile as they lie (the order is the one the 32-row fragment reads want: conflict free without
// a swizzle).  Four to six LDS stages, the K loop software pipelined by hand as in the finetune task's weight GEMM
// (one wave per SIMD has nobody to hide its waits).  Rows and tiles that do not exist, and stages past the end of the
// range, are loaded from an offset outside the buffer resource, which the hardware answers with zeros.
#include "decode_large.h"

#include <algorithm>
#include <mutex>

#include "device_utils.h"

namespace harli {
namespace {

constexpr int BK = 32, BN = 256, NT = 256;
constexpr int BSZ = BN * BK * 2;  // 16 KiB: one stage of the weight side
constexpr int ER = (128 + 8) * 4;  // staged row of the epilogue in bytes
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct DgemmArgs {
  const unsigned short* x;         // [x_tiles][steps][64][8]
  int x_tiles, steps;
  const unsigned short *w0, *w1;   // [w_tiles16][steps][64][8]; w1: the second matrix of a pair or null
  int w_tiles16;                   // 16-row tiles of one matrix
  int tiles_n1, tiles_n;           // 256-row tiles of one matrix, of all matrices
  int tiles_m, ksplit, Mpad;
  float* part;                     // [ksplit][Mpad][tiles_n * 256]
};

#define DG_WAITV(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
#define DG_SB0() __builtin_amdgcn_sched_barrier(0)
#define DG_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// LDS stages: the weights come from HBM, whose latency under load is several K steps long, so the ring is as deep as
// 160 KiB of LDS allow (bytes in flight per compute unit are what the stream's rate follows).
template <int FM>
constexpr int dg_stages() { return FM <= 2 ? 6 : FM == 3 ? 5 : 4; }

template <int FM>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, 1))) k_dgemm(DgemmArgs a) {
  constexpr int BM = 64 * FM, ASZ = BM * BK * 2, STG = ASZ + BSZ, NS = dg_stages<FM>();
  constexpr int LOADS = FM + 4;  // direct-to-LDS loads a wave issues per stage
  static_assert(4 * 32 * ER <= NS * STG, "epilogue staging must fit the stage buffers");
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;  // 2 x 2 waves of (32 FM) x 128
  int w = blockIdx.x;
  const int tn = w % a.tiles_n;
  w /= a.tiles_n;
  const int tm = w % a.tiles_m, split = w / a.tiles_m;
  if (split >= a.ksplit) return;
  const int s_begin = (int)((long long)a.steps * split / a.ksplit);
  const int n_stage = (int)((long long)a.steps * (split + 1) / a.ksplit) - s_begin;
  const int n_step = (n_stage + NS - 1) / NS * NS;  // the loop body covers NS stages; stages past the end multiply zeros

  f32x16 acc[FM][4];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Loads: instruction j of a wave copies one 16 x 32 tile (1 KiB, lane l its 16 bytes at 16 l) to LDS as it lies in
  // memory: fragment order, chunk c (8 k) of row r at (16 c + r) * 16.  Consecutive lanes read consecutive addresses --
  // a permuted assignment (rows of 64 bytes in LDS) was measured at 0.83 us per K step against the 0.37 us its MFMAs
  // take: the lanes of a quad then fall into four cache lines and the address path serialises them.
  // Only the per-lane offset is range checked by the hardware, so whatever must read as zero gets the offset kOut, and
  // the scalar offsets (tile and k step) are kept inside the operand by construction.
  const unsigned vlane = (unsigned)lane * 16u;
  constexpr unsigned kOut = 0x80000000u;
  constexpr int kRsrcFlags = 0x00020000;  // raw buffer of dwords
  const bool second = tn >= a.tiles_n1;
  const unsigned short* wp = second ? a.w1 : a.w0;
  const int tn1 = second ? tn - a.tiles_n1 : tn;
  const unsigned tile_bytes = (unsigned)a.steps * 1024u;
  __amdgpu_buffer_rsrc_t rsA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(a.x), 0, (int)((unsigned)a.x_tiles * tile_bytes), kRsrcFlags);
  __amdgpu_buffer_rsrc_t rsB =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(wp), 0, (int)((unsigned)a.w_tiles16 * tile_bytes), kRsrcFlags);
  unsigned voffA[FM], voffB[4], soffB[4];
#pragma unroll
  for (int j = 0; j < FM; ++j) {
    const int bt = tm * (BM / 16) + wave * FM + j;  // 16-row batch tile
    voffA[j] = bt < a.x_tiles ? (unsigned)bt * tile_bytes + vlane : kOut;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int t16 = tn1 * 16 + wave * 4 + j;  // 16-row weight tile
    const bool ok = t16 < a.w_tiles16;
    voffB[j] = ok ? vlane : kOut;
    soffB[j] = ((unsigned)(ok ? t16 : 0) * (unsigned)a.steps + (unsigned)s_begin) * 1024u;
  }
  unsigned soffA = (unsigned)s_begin * 1024u;
  int issued = 0;
  bool valid = n_stage > 0;

#define DG_ADVANCE()                                                       \
  do {                                                                     \
    ++issued;                                                              \
    valid = issued < n_stage;                                              \
    if (valid) {                                                           \
      soffA += 1024u;                                                      \
      _Pragma("unroll") for (int j = 0; j < 4; ++j) soffB[j] += 1024u;    \
    }                                                                      \
  } while (0)
#define DG_BL(rs, voff, soff, sp) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(sp), 16, (int)(voff), (int)(soff), 0, 0)
#define DG_ISSUE(buf)                                                                                              \
  do {                                                                                                             \
    char* SA = smem + (buf) * STG;                                                                                 \
    char* SB = SA + ASZ;                                                                                           \
    _Pragma("unroll") for (int j = 0; j < FM; ++j) DG_BL(rsA, valid ? voffA[j] : kOut, soffA, SA + (wave * FM + j) * 1024); \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) DG_BL(rsB, valid ? voffB[j] : kOut, soffB[j], SB + (wave * 4 + j) * 1024); \
  } while (0)

  // fragment reads of a 32-row block (two tiles, 2 KiB): row lane%32, chunk 2 sub + lane/32.  Sixteen lanes read 256
  // contiguous bytes: conflict free as the tiles lie.
  const int fo0 = ((lane & 31) >> 4) * 1024 + ((lane >> 5) * 16 + (lane & 15)) * 16;
  const int fo1 = fo0 + 512;
  const int aoff = wm * (FM * 32) * 64, boff = ASZ + wn * 128 * 64;
  u32x4 fa0[FM], fb0[4], fa1[FM], fb1[4];
#define DG_RD(FA, FB, buf, sub)                                                                                    \
  do {                                                                                                             \
    const char* sa_ = smem + (buf) * STG + aoff + ((sub) ? fo1 : fo0);                                             \
    const char* sb_ = smem + (buf) * STG + boff + ((sub) ? fo1 : fo0);                                             \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) FA[i] = *reinterpret_cast<const u32x4*>(sa_ + i * 2048);        \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) FB[j] = *reinterpret_cast<const u32x4*>(sb_ + j * 2048);         \
  } while (0)
#define DG_MM(FA, FB)                                                                                              \
  do {                                                                                                             \
    _Pragma("unroll") for (int i = 0; i < FM; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)                   \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, FA[i]),                     \
                                                            __builtin_bit_cast(bf16x8, FB[j]), acc[i][j], 0, 0, 0); \
  } while (0)
  // issue order of a half step: the fragment reads ride on the first MFMAs, then one load per MFMA
  constexpr int kRd = (FM + 4) / 2;
  constexpr int kRest = 4 * FM - kRd;
  constexpr int kLd = LOADS < kRest ? LOADS : kRest;
#define DG_PIPE_RD()                                                                            \
  do {                                                                                          \
    _Pragma("unroll") for (int q = 0; q < kRd; ++q) { DG_SGB(0x008, 1); DG_SGB(0x100, 2); }     \
  } while (0)
#define DG_PIPE1()          \
  do {                      \
    DG_PIPE_RD();           \
    DG_SGB(0x008, kRest);   \
  } while (0)
#define DG_PIPE2()                                                                              \
  do {                                                                                          \
    DG_PIPE_RD();                                                                               \
    _Pragma("unroll") for (int q = 0; q < kLd; ++q) { DG_SGB(0x008, 1); DG_SGB(0x020, 1); }     \
    if (LOADS > kLd) DG_SGB(0x020, LOADS - kLd);                                                \
    if (kRest > kLd) DG_SGB(0x008, kRest - kLd);                                                \
  } while (0)
#define DG_STEP(cur, nxt, dma)                                                                   \
  do {                                                                                           \
    DG_RD(fa1, fb1, cur, 1);                                                                     \
    DG_MM(fa0, fb0);                                                                             \
    DG_PIPE1();                                                                                  \
    DG_SB0();                                                                                    \
    DG_ADVANCE();                                                                                \
    DG_WAITV((NS - 3) * LOADS); /* all but the NS - 3 newest stages in flight have landed */    \
    __builtin_amdgcn_s_barrier();                                                                \
    DG_SB0();                                                                                    \
    DG_RD(fa0, fb0, nxt, 0);                                                                     \
    DG_ISSUE(dma);                                                                               \
    DG_MM(fa1, fb1);                                                                             \
    DG_PIPE2();                                                                                  \
    DG_SB0();                                                                                    \
  } while (0)

  if (n_stage > 0) {
#pragma unroll
    for (int i = 0; i < NS - 1; ++i) {
      if (i > 0) DG_ADVANCE();
      DG_ISSUE(i);
    }
    DG_WAITV((NS - 2) * LOADS);
    __builtin_amdgcn_s_barrier();
    DG_RD(fa0, fb0, 0, 0);
    DG_SB0();
    for (int st = 0; st < n_step; st += NS) {
#pragma unroll
      for (int i = 0; i < NS; ++i) DG_STEP(i, (i + 1) % NS, (i + NS - 1) % NS);
    }
    DG_WAITV(0);
  }
  __syncthreads();  // every wave is done with the stage buffers: the epilogue reuses them
#undef DG_ADVANCE
#undef DG_BL
#undef DG_ISSUE
#undef DG_RD
#undef DG_MM
#undef DG_PIPE_RD
#undef DG_PIPE1
#undef DG_PIPE2
#undef DG_STEP

  // ---- the partial tile: staged per 32-row slab so that a row leaves as 512 contiguous bytes -----------------------
  // a lane of accumulator j holds rows 8 (v/4) + 4 (lane/32) + v%4 of column lane%32 of that 32 x 32 block
  char* ebuf = smem + wave * (32 * ER);
  const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
  const size_t ncols = (size_t)a.tiles_n * BN;
  float* prow = a.part + ((size_t)split * a.Mpad + (size_t)tm * BM + wm * (FM * 32)) * ncols + (size_t)tn * BN + wn * 128;
  const int c4 = (lane & 31) * 4;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        *reinterpret_cast<float*>(ebuf + (8 * (v >> 2) + rgrp + (v & 3)) * ER + (j * 32 + col_l) * 4) = acc[i][j][v];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int row = it * 2 + (lane >> 5);
      const float4 o = *reinterpret_cast<const float4*>(ebuf + row * ER + c4 * 4);
      *reinterpret_cast<float4*>(prow + (size_t)(i * 32 + row) * ncols + c4) = o;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// Sum over the K ranges of four consecutive columns of batch row b, in range order.
__device__ __forceinline__ float4 part_sum4(const float* part, int ksplit, size_t split_stride, size_t off) {
  float4 s = *reinterpret_cast<const float4*>(part + off);
  for (int sp = 1; sp < ksplit; ++sp) {
    const float4 v = *reinterpret_cast<const float4*>(part + (size_t)sp * split_stride + off);
    s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
  }
  return s;
}

// x1 = res + sum, the next operand bf16(x1 * g) in fragment order, and this 16-column tile's share of sum x1^2.
// Thread: four columns of one batch row; the four threads of a tile are neighbours in a wave.
__global__ void __launch_bounds__(256) k_dg_resid(SkinnyArgs a, const float* part, int ksplit, size_t split_stride, size_t ncols) {
  const int b = blockIdx.y, n0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  const bool active = n0 < a.n_rows;  // n_rows is a multiple of 8, so the four columns are all in or all out
  float s2 = 0.f;
  if (active) {
    const float4 s = part_sum4(part, ksplit, split_stride, (size_t)b * ncols + n0);
    const float4 rs = *reinterpret_cast<const float4*>(a.res + (size_t)b * a.n_rows + n0);
    const float o0 = rs.x + s.x, o1 = rs.y + s.y, o2 = rs.z + s.z, o3 = rs.w + s.w;
    *reinterpret_cast<float4*>(a.out + (size_t)b * a.n_rows + n0) = make_float4(o0, o1, o2, o3);
    if (a.hxn) {
      const float4 gn = *reinterpret_cast<const float4*>(a.gnext + n0);
      *reinterpret_cast<uint2*>(a.hxn + xfrag_off(b, n0, (a.n_rows + 31) >> 5)) =
          make_uint2(pack_bf2(o0 * gn.x, o1 * gn.y), pack_bf2(o2 * gn.z, o3 * gn.w));
    }
    s2 = (o0 * o0 + o1 * o1) + (o2 * o2 + o3 * o3);
  }
  s2 += __shfl_xor(s2, 1, 64);
  s2 += __shfl_xor(s2, 2, 64);
  if (active && (threadIdx.x & 3) == 0 && a.ssq_out) a.ssq_out[(size_t)b * a.ssq_np + (n0 >> 4)] = s2;
}

// m = silu(rho * gate) * (rho * up) as the next operand in fragment order.
__global__ void __launch_bounds__(256) k_dg_gateup(SkinnyArgs a, const float* part, int ksplit, size_t split_stride, size_t ncols,
                                                   int up_col0) {
  const int b = blockIdx.y;
  // every wave adds up the row's norm for itself (a few KB from L2); a workgroup then takes several groups of 1024
  // columns so that this is paid once per 4096 columns
  const float rho = rsqrtf(ssq_row_sum(a.ssq_in + (size_t)b * a.ssq_np, a.ssq_np, (threadIdx.x & 63) >> 4) * a.inv_dim + a.eps);
  const int steps_n = (a.n_rows + 31) >> 5;
  for (int n0 = (blockIdx.x * 256 + threadIdx.x) * 4; n0 < a.n_rows; n0 += gridDim.x * 1024) {
    const float4 ga = part_sum4(part, ksplit, split_stride, (size_t)b * ncols + n0);
    const float4 up = part_sum4(part, ksplit, split_stride, (size_t)b * ncols + up_col0 + n0);
    const float gv[4] = {ga.x * rho, ga.y * rho, ga.z * rho, ga.w * rho}, uv[4] = {up.x * rho, up.y * rho, up.z * rho, up.w * rho};
    float m[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) m[e] = gv[e] / (1.f + __expf(-gv[e])) * uv[e];
    *reinterpret_cast<uint2*>(a.mbuf + xfrag_off(b, n0, steps_n)) = make_uint2(pack_bf2(m[0], m[1]), pack_bf2(m[2], m[3]));
  }
}

// logits = rho * sum (the output layer after the last layer's norm)
__global__ void __launch_bounds__(256) k_dg_lm(SkinnyArgs a, const float* part, int ksplit, size_t split_stride, size_t ncols) {
  const int b = blockIdx.y;
  const float rho = rsqrtf(ssq_row_sum(a.ssq_in + (size_t)b * a.ssq_np, a.ssq_np, (threadIdx.x & 63) >> 4) * a.inv_dim + a.eps);
  const bool vec = (a.n_rows & 3) == 0;  // rows of the logits are 16-byte aligned
  for (int n0 = (blockIdx.x * 256 + threadIdx.x) * 4; n0 < a.n_rows; n0 += gridDim.x * 1024) {
    const float4 s = part_sum4(part, ksplit, split_stride, (size_t)b * ncols + n0);  // the partial rows are padded to whole tiles
    float* o = a.logits + (size_t)b * a.n_rows + n0;
    if (vec) {
      *reinterpret_cast<float4*>(o) = make_float4(s.x * rho, s.y * rho, s.z * rho, s.w * rho);
    } else {
      const float v[4] = {s.x * rho, s.y * rho, s.z * rho, s.w * rho};
      for (int e = 0; e < 4 && n0 + e < a.n_rows; ++e) o[e] = v[e];
    }
  }
}

// q, k, v = rho * sum + bias; rotary embedding on q and k; q to the attention's query buffer, k and v to the page the
// sequence's next token belongs in.  Thread: rotation indices idx0..idx0+3 (and their partners d/2 further) of one head.
__global__ void __launch_bounds__(256) k_dg_qkv(SkinnyArgs a, const float* part, int ksplit, size_t split_stride, size_t ncols) {
  const int b = blockIdx.y, t = blockIdx.x * 256 + threadIdx.x;
  const float rho = rsqrtf(ssq_row_sum(a.ssq_in + (size_t)b * a.ssq_np, a.ssq_np, (threadIdx.x & 63) >> 4) * a.inv_dim + a.eps);
  const int half = a.d >> 1, per_head = half >> 2;
  const int head = t / per_head, idx0 = (t - head * per_head) * 4;
  if (head >= a.n_q + 2 * a.n_kv) return;
  int which, hl;
  if (head < a.n_q) {
    which = 0, hl = head;
  } else if (head < a.n_q + a.n_kv) {
    which = 1, hl = head - a.n_q;
  } else {
    which = 2, hl = head - a.n_q - a.n_kv;
  }
  // q, k and v are packed as one matrix with heads in the order q.., k.., v..
  const size_t col0 = (size_t)b * ncols + (size_t)head * a.d + idx0;
  const float4 s0 = part_sum4(part, ksplit, split_stride, col0), s1 = part_sum4(part, ksplit, split_stride, col0 + half);
  float4 b0 = make_float4(0.f, 0.f, 0.f, 0.f), b1 = b0;
  if (a.bias[which]) {
    const float* bp = a.bias[which] + hl * a.d + idx0;
    b0 = *reinterpret_cast<const float4*>(bp);
    b1 = *reinterpret_cast<const float4*>(bp + half);
  }
  const float v0[4] = {s0.x * rho + b0.x, s0.y * rho + b0.y, s0.z * rho + b0.z, s0.w * rho + b0.w};
  const float v1[4] = {s1.x * rho + b1.x, s1.y * rho + b1.y, s1.z * rho + b1.z, s1.w * rho + b1.w};
  float r0[4], r1[4];
  if (which != 2) {
    const float* cs = a.rope + ((size_t)b * half + idx0) * 2;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float c = cs[2 * e], s = cs[2 * e + 1];
      r0[e] = v0[e] * c - v1[e] * s;
      r1[e] = v1[e] * c + v0[e] * s;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) r0[e] = v0[e], r1[e] = v1[e];
  }
  if (which == 0) {
    float* q = a.qbuf + (size_t)b * (a.n_q * a.d) + hl * a.d + idx0;
    *reinterpret_cast<float4*>(q) = make_float4(r0[0], r0[1], r0[2], r0[3]);
    *reinterpret_cast<float4*>(q + half) = make_float4(r1[0], r1[1], r1[2], r1[3]);
    return;
  }
  const int n = a.kv_len[b];
  const int lp = n / a.geom.page_tokens, slot = n - lp * a.geom.page_tokens;
  const int page = (n >= 0 && lp < a.max_pages) ? a.page_table[(size_t)b * a.max_pages + lp] : -1;
  if (page < 0 || page >= a.geom.n_pages_total) {
    if (idx0 == 0) atomicOr(a.err_flag, 1);
    return;
  }
  // inside a page the order is [kv head][token slot][head_dim]
  char* base = a.slab + kv_page_off(a.geom, page, a.layer, which - 1) + ((size_t)(hl * a.geom.page_tokens + slot) * a.d) * sizeof(unsigned short);
  unsigned short* dst = reinterpret_cast<unsigned short*>(base) + idx0;
  *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf2(r0[0], r0[1]), pack_bf2(r0[2], r0[3]));
  *reinterpret_cast<uint2*>(dst + half) = make_uint2(pack_bf2(r1[0], r1[1]), pack_bf2(r1[2], r1[3]));
}

template <int FM>
constexpr int dg_lds_bytes() { return dg_stages<FM>() * (64 * FM * BK * 2 + BSZ); }

std::once_flag g_attr_once;
hipError_t g_attr_err = hipSuccess;
int g_force_ksplit = 0;  // measurement hook: ranges of K whatever the cost model says

}  // namespace

void dg_force_ksplit(int ksplit) { g_force_ksplit = ksplit > 0 ? ksplit : 0; }

// Smallest batch on the tiled path.  Measured on the 7B/8B-class models at full depth: at 48 and 64 sequences the
// tiled step is 9-24 % shorter than the pass-wise one, at 24 and 32 it is 1-3 % longer.
constexpr int kMinBatch = 33;
int g_min_batch = kMinBatch;
void dg_set_min_batch(int b) { g_min_batch = b > 0 ? b : kMinBatch; }
int dg_min_batch() { return g_min_batch; }

DgPlan dg_plan(int B, int n_rows, int n_mat, int K, int n_cu, size_t ws_bytes) {
  DgPlan p{};
  p.FM = B <= 64 ? 1 : B <= 128 ? 2 : B <= 192 ? 3 : 4;
  const int BM = 64 * p.FM;
  p.tiles_m = (B + BM - 1) / BM;
  p.Mpad = p.tiles_m * BM;
  p.tiles_n = ((n_rows + BN - 1) / BN) * n_mat;
  const int steps = (K + BK - 1) / BK, T = p.tiles_m * p.tiles_n;
  if (n_cu < 1) n_cu = 1;
  // Cost of a cut in microseconds, fitted to measurements on 256 compute units (it picks within 2 us of the best cut
  // measured for every GEMM of the 7B- and 8B-class layers at 96 to 256 sequences).  A K step of a workgroup takes
  // 0.36 / 0.47 / 0.60 us at 128 / 192 / 256 batch rows when it has the memory system to itself (the pace of one wave
  // per SIMD) and up to 0.35 us more as the workgroups running together fill the chip (weights from HBM, the batch
  // operand from L2); a round of workgroups adds about 7 us of filling and draining; every range adds a partial
  // matrix that is written once and read once (0.30 us per MB).
  // Ranges shorter than two passes of the stage ring are not worth a workgroup.
  const double t_wg = p.FM == 1 ? 0.30 : p.FM == 2 ? 0.36 : p.FM == 3 ? 0.47 : 0.60, t_fixed = 7.0, t_part_mb = 0.30;
  const int ks_max = std::max(1, std::min(32, steps / 8));
  double best = -1.0;
  for (int ks = 1; ks <= ks_max; ++ks) {
    const size_t bytes = (size_t)ks * p.Mpad * p.tiles_n * BN * 4;
    if (bytes > ws_bytes) break;
    const int rounds = (T * ks + n_cu - 1) / n_cu;
    const double busy = std::min(T * ks, n_cu) / 256.0;
    const double t_step = t_wg + 0.35 * busy * busy;
    const double cost = rounds * (((steps + ks - 1) / ks) * t_step + t_fixed) + (double)bytes / 1048576.0 * t_part_mb;
    if (best < 0 || cost < best || ks == g_force_ksplit) best = cost, p.ksplit = ks, p.rounds = rounds, p.part_bytes = bytes;
    if (ks == g_force_ksplit) break;
  }
  return p;  // ksplit 0: not even one range fits the workspace
}

size_t dg_workspace_bytes(const harli_model_cfg& m, int n_cu) {
  if (m.dtype != HARLI_BF16 || m.max_batch < 17) return 0;  // 17: the lowest setting of the measurement hook
  const int QKV = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim, QD = m.n_q_heads * m.head_dim;
  size_t need = 0;
  const int bs[5] = {64, 128, 192, 256, m.max_batch};
  for (int B : bs) {
    if (B > m.max_batch) continue;
    need = std::max(need, dg_plan(B, QKV, 1, m.hidden, n_cu, ~size_t(0)).part_bytes);
    need = std::max(need, dg_plan(B, m.hidden, 1, QD, n_cu, ~size_t(0)).part_bytes);
    need = std::max(need, dg_plan(B, m.ffn, 2, m.hidden, n_cu, ~size_t(0)).part_bytes);
    need = std::max(need, dg_plan(B, m.hidden, 1, m.ffn, n_cu, ~size_t(0)).part_bytes);
    if (m.vocab > 0) need = std::max(need, dg_plan(B, m.vocab, 1, m.hidden, n_cu, ~size_t(0)).part_bytes);
  }
  return std::min(need, (size_t)192 << 20);
}

// The tile kernels need more dynamic LDS than the default limit; set once per process (harli_ctx_create calls this when
// it takes the workspace, so that no step -- a captured one included -- is the first to ask).
harli_status dg_init() {
  std::call_once(g_attr_once, [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dgemm<1>), hipFuncAttributeMaxDynamicSharedMemorySize, dg_lds_bytes<1>());
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dgemm<2>), hipFuncAttributeMaxDynamicSharedMemorySize, dg_lds_bytes<2>());
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dgemm<3>), hipFuncAttributeMaxDynamicSharedMemorySize, dg_lds_bytes<3>());
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_dgemm<4>), hipFuncAttributeMaxDynamicSharedMemorySize, dg_lds_bytes<4>());
    g_attr_err = e;
  });
  HARLI_HIP(g_attr_err);
  return HARLI_OK;
}

harli_status dg_gemm(DgKind kind, const SkinnyArgs& a, int x_tiles, float* part, size_t part_bytes, int n_cu, hipStream_t st, DgPlan* used) {
  {
    harli_status rc = dg_init();
    if (rc != HARLI_OK) return rc;
  }
  const int n_mat = kind == DG_GATEUP ? 2 : 1;
  const int n_rows = kind == DG_QKV ? (a.n_q + 2 * a.n_kv) * a.d : a.n_rows;
  const int steps = (a.K + BK - 1) / BK, w_tiles16 = (n_rows + 15) / 16;
  if (!part || a.B < 1 || x_tiles * 16 < a.B || (kind == DG_GATEUP && !a.w1))
    return fail(HARLI_ERR_INVALID, "decode (large batch): bad arguments (batch %d, %d operand tiles)", a.B, x_tiles);
  if ((kind != DG_LM && (a.n_rows & 7)) || (kind == DG_QKV && (a.d & 15)))
    return fail(HARLI_ERR_INVALID, "decode (large batch): %d output rows, head size %d", a.n_rows, a.d);
  // the kernel addresses both operands with 32-bit byte offsets below 2^31
  if ((long long)(w_tiles16 + 16) * steps * 1024 >= (1ll << 31) || (long long)x_tiles * steps * 1024 >= (1ll << 31))
    return fail(HARLI_ERR_INVALID, "decode (large batch): an operand of 2 GiB or more (%d rows, K %d)", n_rows, a.K);
  const DgPlan p = dg_plan(a.B, n_rows, n_mat, a.K, n_cu, part_bytes);
  if (p.ksplit < 1) return fail(HARLI_ERR_INVALID, "decode (large batch): a workspace of %zu bytes cannot hold one partial matrix", part_bytes);
  DgemmArgs g{};
  g.x = a.x;
  g.x_tiles = x_tiles;
  g.steps = steps;
  g.w0 = a.w0;
  g.w1 = n_mat == 2 ? a.w1 : nullptr;
  g.w_tiles16 = w_tiles16;
  g.tiles_n1 = p.tiles_n / n_mat;
  g.tiles_n = p.tiles_n;
  g.tiles_m = p.tiles_m;
  g.ksplit = p.ksplit;
  g.Mpad = p.Mpad;
  g.part = part;
  const dim3 grid((unsigned)(p.tiles_n * p.tiles_m * p.ksplit));
  if (p.FM == 1) hipLaunchKernelGGL(k_dgemm<1>, grid, dim3(NT), dg_lds_bytes<1>(), st, g);
  else if (p.FM == 2) hipLaunchKernelGGL(k_dgemm<2>, grid, dim3(NT), dg_lds_bytes<2>(), st, g);
  else if (p.FM == 3) hipLaunchKernelGGL(k_dgemm<3>, grid, dim3(NT), dg_lds_bytes<3>(), st, g);
  else hipLaunchKernelGGL(k_dgemm<4>, grid, dim3(NT), dg_lds_bytes<4>(), st, g);
  HARLI_HIP(hipGetLastError());
  *used = p;
  return HARLI_OK;
}

harli_status dg_epilogue(DgKind kind, const SkinnyArgs& a, const DgPlan& p, const float* part, hipStream_t st) {
  const size_t ncols = (size_t)p.tiles_n * BN, split_stride = (size_t)p.Mpad * ncols;
  if (kind == DG_RESID) {
    hipLaunchKernelGGL(k_dg_resid, dim3((unsigned)((a.n_rows / 4 + 255) / 256), (unsigned)a.B), dim3(256), 0, st, a, part, p.ksplit, split_stride, ncols);
  } else if (kind == DG_GATEUP) {
    hipLaunchKernelGGL(k_dg_gateup, dim3((unsigned)((a.n_rows + 4095) / 4096), (unsigned)a.B), dim3(256), 0, st, a, part, p.ksplit, split_stride, ncols,
                       (p.tiles_n / 2) * BN);
  } else if (kind == DG_LM) {
    hipLaunchKernelGGL(k_dg_lm, dim3((unsigned)((a.n_rows + 4095) / 4096), (unsigned)a.B), dim3(256), 0, st, a, part, p.ksplit, split_stride, ncols);
  } else {
    const int threads = (a.n_q + 2 * a.n_kv) * (a.d / 8);
    hipLaunchKernelGGL(k_dg_qkv, dim3((unsigned)((threads + 255) / 256), (unsigned)a.B), dim3(256), 0, st, a, part, p.ksplit, split_stride, ncols);
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

harli_status dg_launch(DgKind kind, const SkinnyArgs& a, int x_tiles, float* part, size_t part_bytes, int n_cu, hipStream_t st) {
  DgPlan p{};
  harli_status rc = dg_gemm(kind, a, x_tiles, part, part_bytes, n_cu, st, &p);
  if (rc != HARLI_OK) return rc;
  return dg_epilogue(kind, a, p, part, st);
}

}  // namespace harli
