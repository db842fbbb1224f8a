// Decode step for gfx950 (Harli Sec. 2.1: one new token per sequence per step,
// reusing the KV cache; Sec. 2.2.1: the step is bound by DRAM bandwidth -- its
// GEMMs have M = batch -- so every kernel here is built around streaming the
// weights and the paged KV cache from HBM exactly once, in 1 KiB contiguous
// wavefront loads).
//
// Per layer, bf16 storage:
//   skinny<QKV>     h W{q,k,v}^T, x rho, rotary embedding, q -> workspace, k/v -> KV pages
//   paged_attn      split-KV attention over the page table (+ a small merge launch)
//   skinny<RESID>   x1 = x + o Wo^T, next operand bf16(x1*g2), sum x1^2
//   skinny<GATEUP>  m = silu(rho h2 Wg^T) * (rho h2 Wu^T)
//   skinny<RESID>   y = x1 + m Wd^T, operand and sum of squares for the next layer
// RMSNorm is folded: the GEMM operand is bf16(x*g) and the per-row factor
// rho = rsqrt(mean x^2 + eps) multiplies the fp32 accumulator afterwards.
//
// The skinny GEMM keeps the batch (<= 64 rows per pass) as the MFMA "column"
// operand and streams 16-row weight tiles as the "row" operand of
// v_mfma_f32_16x16x32_bf16.  Both operands are stored in MFMA fragment order
// (the decode instance keeps a pre-shuffled private copy of the frozen weights,
// as the paper's inference instance keeps its own copy, Sec. 7): a 16 x 32 tile
// is 64 lanes x 16 bytes, contiguous, so a wavefront load is one 1 KiB burst and
// needs no LDS staging.  Address-scattered 16-byte loads (16 rows per
// instruction) were measured at 3.6 TB/s against 5.0 TB/s for this layout.
// A workgroup is TW tiles x KW waves; the KW waves split K and reduce through
// LDS, so epilogues see complete sums.
#include <mutex>

#include "ctx.h"
#include "decode_large.h"
#include "device_utils.h"
#include "gemm2.h"

using namespace harli;

namespace {

constexpr int kPageTokens = 16;
constexpr int kComputeUnits = 256;  // MI355X; only steers a tiling choice

enum { MODE_QKV = 0, MODE_RESID = 1, MODE_GATEUP = 2, MODE_LM = 3 };

__device__ __forceinline__ uint4 ld16(const unsigned short* p) { return *reinterpret_cast<const uint4*>(p); }

// RT = 16-row weight tiles per wave: a wave holds RT x NB accumulator tiles, so that a batch fragment fetched for a
// k-step serves RT weight fragments (at 64 batch rows every wave otherwise pulls four batch fragments through the
// vector cache for each weight fragment it streams).  RT = 1 for small batches, where the weights are the traffic.
template <int MODE, int NB, int TW, int KW, int U, int RT>
__global__ void __launch_bounds__(TW * KW * 64) k_skinny(SkinnyArgs a) {
  constexpr int WAVES = TW * KW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int t_w = wave / KW, ks = wave - t_w * KW;
  const int wg = blockIdx.x;
  const int steps = (a.K + 31) >> 5;
  const int n_tiles = (a.n_rows + 15) >> 4;  // 16-row tiles of the (unpacked) output

  // ---- which 16-row weight tiles this workgroup covers: tile_row0(t, r), t < TW, r < RT ----------
  int which = 0, hl = 0, pg = 0;  // QKV bookkeeping (uniform over the workgroup)
  const int half = a.d >> 1;
  if (MODE == MODE_QKV) {
    const int ppg = (half >> 4) / RT;  // workgroups per head: the d/2 rotation indices in groups of 16 * RT
    const int head = wg / ppg;
    pg = wg - head * ppg;
    if (head < a.n_q) {
      which = 0; hl = head;
    } else if (head < a.n_q + a.n_kv) {
      which = 1; hl = head - a.n_q;
    } else {
      which = 2; hl = head - a.n_q - a.n_kv;
    }
  }
  // first output row (within its projection) of tile (t, r)
  auto tile_row0 = [&](int t, int r) -> int {
    if (MODE == MODE_QKV) return hl * a.d + t * half + (pg * RT + r) * 16;
    if (MODE == MODE_GATEUP) return (wg * RT + r) * 16;
    return ((wg * TW + t) * RT + r) * 16;
  };
  const unsigned short* wt[RT];
  bool tile_ok[RT];
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    int tile;  // index of the 16-row tile in the packed matrix this wave reads
    if (MODE == MODE_QKV) {
      // q, k and v are packed as one matrix with heads in the order q.., k.., v..
      const int head = which == 0 ? hl : which == 1 ? a.n_q + hl : a.n_q + a.n_kv + hl;
      tile = (head * a.d + t_w * half + (pg * RT + r) * 16) >> 4;
      tile_ok[r] = true;
    } else {
      tile = MODE == MODE_GATEUP ? wg * RT + r : (wg * TW + t_w) * RT + r;
      tile_ok[r] = tile < n_tiles;
      if (!tile_ok[r]) tile = 0;  // past the last tile: read tile 0 (in bounds), the result is never stored
    }
    const unsigned short* base = (MODE == MODE_GATEUP && t_w != 0) ? a.w1 : a.w0;
    wt[r] = base + ((size_t)tile * steps * 64 + lane) * 8;
  }

  const unsigned short* xf0[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) xf0[nb] = a.x + (((size_t)((a.b0 >> 4) + nb) * steps) * 64 + lane) * 8;

  f32x4 acc[RT][NB];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[r][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- epilogue operands are fetched now, so that the epilogue issues no dependent load ----
  const bool epi = wave < NB;  // wave nb finishes batch tile nb
  const int jb = a.b0 + wave * 16 + i16;
  const bool active = epi && jb < a.B;
  float pre_ssq = 1.f;
  float2 pre_cs[RT][4];
  float4 pre_res[RT], pre_g[RT];
  int pre_page = -1, pre_slot = 0;
  float4 pre_b0[RT], pre_b1[RT];  // biases of the two half tiles
#pragma unroll
  for (int r = 0; r < RT; ++r) {
    pre_res[r] = pre_g[r] = pre_b0[r] = pre_b1[r] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int e = 0; e < 4; ++e) pre_cs[r][e] = make_float2(1.f, 0.f);
  }
  // The partial sums of squares of this wave's 16 batch rows.  Small batches (NB <= 2, where a step is short enough
  // for a memory round trip to show): the rows are copied to LDS by loads that need no register and no wait here, and
  // are added up after the stream; otherwise they are added now (the wave waits for them once, before its stream).
  constexpr bool kSsqLds = MODE != MODE_RESID && NB <= 2;
  extern __shared__ __attribute__((aligned(1024))) char ssq_lds[];
  const int ssq_stride = (a.ssq_np * 4 + 1023) & ~1023;  // bytes per staged row
  if (MODE != MODE_RESID && epi) {  // whole waves; rows past the batch read row B - 1
    if constexpr (kSsqLds) {
      for (int r = 0; r < 16; ++r) {
        const float* row = a.ssq_in + (size_t)min(a.b0 + wave * 16 + r, a.B - 1) * a.ssq_np;
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(row), 0, a.ssq_np * 4, 0x00020000);
        for (int k = 0; k < ssq_stride; k += 1024)  // lanes past the row are out of the resource's range: zeros
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)(ssq_lds + (wave * 16 + r) * ssq_stride + k),
                                                   16, lane * 16 + k, 0, 0, 0);
      }
    } else {
      pre_ssq = ssq_row_sum(a.ssq_in + (size_t)min(jb, a.B - 1) * a.ssq_np, a.ssq_np, g);
    }
  }
  if (active) {
    if (MODE == MODE_QKV) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        const int idx0 = (pg * RT + r) * 16 + 4 * g;  // rotation index of this lane's first row in tile r
        if (a.bias[which]) {  // rows hl*d + idx0 + e and the same + d/2; d % 32 == 0 keeps them 16-byte aligned
          const float* bp = a.bias[which] + hl * a.d + idx0;
          pre_b0[r] = *reinterpret_cast<const float4*>(bp);
          pre_b1[r] = *reinterpret_cast<const float4*>(bp + half);
        }
        if (which != 2) {
          const float* cs = a.rope + ((size_t)jb * half + idx0) * 2;
#pragma unroll
          for (int e = 0; e < 4; ++e) pre_cs[r][e] = make_float2(cs[2 * e], cs[2 * e + 1]);
        }
      }
      if (which != 0) {
        const int n = a.kv_len[jb];
        const int lp = n / a.geom.page_tokens;
        pre_slot = n - lp * a.geom.page_tokens;
        pre_page = (n >= 0 && lp < a.max_pages)
                       ? a.page_table[(size_t)jb * a.max_pages + lp]
                       : -1;
      }
    }
    if (MODE == MODE_RESID) {
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        const int n0 = tile_row0(0, r) + 4 * g;
        if (n0 < a.n_rows) {
          pre_res[r] = *reinterpret_cast<const float4*>(a.res + (size_t)jb * a.n_rows + n0);
          if (a.hxn) pre_g[r] = *reinterpret_cast<const float4*>(a.gnext + n0);
        }
      }
    }
  }

  // ---- stream: each instruction below reads 1 KiB contiguous per wave ---------------------
  const int s_begin = (int)(((long long)steps * ks) / KW), s_end = (int)(((long long)steps * (ks + 1)) / KW);
  bool any_ok = false;
#pragma unroll
  for (int r = 0; r < RT; ++r) any_ok = any_ok || tile_ok[r];
  if (any_ok) {
    int s = s_begin;
    for (; s + U <= s_end; s += U) {
      uint4 wf[U][RT], xf[U][NB];
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int r = 0; r < RT; ++r) wf[u][r] = ld16(wt[r] + (size_t)(s + u) * 512);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) xf[u][nb] = ld16(xf0[nb] + (size_t)(s + u) * 512);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[r][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[u][r]),
                                                                 __builtin_bit_cast(bf16x8, xf[u][nb]), acc[r][nb], 0, 0, 0);
    }
    for (; s < s_end; ++s) {
      uint4 xf[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) xf[nb] = ld16(xf0[nb] + (size_t)s * 512);
#pragma unroll
      for (int r = 0; r < RT; ++r) {
        const uint4 wf = ld16(wt[r] + (size_t)s * 512);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[r][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf),
                                                               __builtin_bit_cast(bf16x8, xf[nb]), acc[r][nb], 0, 0, 0);
      }
    }
  }

  // ---- per row-tile round r: reduce the K split through LDS, then the epilogue ------------------
  __shared__ float4 red[TW][KW][NB][64];
  static_assert(NB <= WAVES, "one epilogue wave per batch tile");
  float rho = 1.f;
  if constexpr (kSsqLds) {
    if (epi) {  // the same chunks in the same order as ssq_row_sum, from the staged copy
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's own copies have landed
      const float* row = reinterpret_cast<const float*>(ssq_lds + (wave * 16 + i16) * ssq_stride);
      float s = 0.f;
      for (int i = g * 4; i < a.ssq_np; i += 16) {
        const float4 v = *reinterpret_cast<const float4*>(row + i);
        s += (v.x + v.y) + (v.z + v.w);
      }
      s += __shfl_xor(s, 16, 64);
      s += __shfl_xor(s, 32, 64);
      pre_ssq = s;
    }
  }
  if (MODE != MODE_RESID && active) rho = rsqrtf(pre_ssq * a.inv_dim + a.eps);
  const int steps_n = (a.n_rows + 31) >> 5;

#pragma unroll
  for (int r = 0; r < RT; ++r) {
    if (r > 0) __syncthreads();  // the readers of the previous round are done with `red`
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      red[t_w][ks][nb][lane] = make_float4(acc[r][nb][0], acc[r][nb][1], acc[r][nb][2], acc[r][nb][3]);
    __syncthreads();
    if (!epi) continue;

    const int nb = wave;
    float v[TW][4];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
      float4 sacc = red[t][0][nb][lane];
#pragma unroll
      for (int w = 1; w < KW; ++w) {
        const float4 o = red[t][w][nb][lane];
        sacc.x += o.x; sacc.y += o.y; sacc.z += o.z; sacc.w += o.w;
      }
      v[t][0] = sacc.x; v[t][1] = sacc.y; v[t][2] = sacc.z; v[t][3] = sacc.w;
    }
    // this lane holds output rows tile_row0(t, r) + 4g + {0..3} of batch entry jb

    if (MODE == MODE_QKV) {
      if (active) {
        const int idx0 = (pg * RT + r) * 16 + 4 * g;  // rotation index of v[.][0]
        float r0[4], r1[4];
        const float b0[4] = {pre_b0[r].x, pre_b0[r].y, pre_b0[r].z, pre_b0[r].w};
        const float b1[4] = {pre_b1[r].x, pre_b1[r].y, pre_b1[r].z, pre_b1[r].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a0 = v[0][e] * rho + b0[e], a1 = v[TW - 1][e] * rho + b1[e];
          if (which != 2) {
            const float2 cs = pre_cs[r][e];
            r0[e] = a0 * cs.x - a1 * cs.y;
            r1[e] = a1 * cs.x + a0 * cs.y;
          } else {
            r0[e] = a0;
            r1[e] = a1;
          }
        }
        if (which == 0) {
          float* q = a.qbuf + (size_t)jb * (a.n_q * a.d) + hl * a.d + idx0;
          *reinterpret_cast<float4*>(q) = make_float4(r0[0], r0[1], r0[2], r0[3]);
          *reinterpret_cast<float4*>(q + half) = make_float4(r1[0], r1[1], r1[2], r1[3]);
        } else {
          const int page = pre_page, slot = pre_slot;
          if (page < 0 || page >= a.geom.n_pages_total) {
            if (g == 0 && r == 0) atomicOr(a.err_flag, 1);
          } else {
            // inside a page the order is [kv head][token slot][head_dim]
            char* base = a.slab + kv_page_off(a.geom, page, a.layer, which - 1) +
                         ((size_t)(hl * a.geom.page_tokens + slot) * a.d) * sizeof(unsigned short);
            unsigned short* dst = reinterpret_cast<unsigned short*>(base) + idx0;
            *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf2(r0[0], r0[1]), pack_bf2(r0[2], r0[3]));
            *reinterpret_cast<uint2*>(dst + half) = make_uint2(pack_bf2(r1[0], r1[1]), pack_bf2(r1[2], r1[3]));
          }
        }
      }
    } else if (MODE == MODE_RESID) {
      const int n0 = tile_row0(0, r) + 4 * g;
      float s2 = 0.f;
      if (active && n0 < a.n_rows) {  // n_rows is a multiple of 8, so the four rows are all in or all out
        const float4 rs = pre_res[r];
        const float o0 = rs.x + v[0][0], o1 = rs.y + v[0][1], o2 = rs.z + v[0][2], o3 = rs.w + v[0][3];
        *reinterpret_cast<float4*>(a.out + (size_t)jb * a.n_rows + n0) = make_float4(o0, o1, o2, o3);
        if (a.hxn) {
          const float4 gn = pre_g[r];
          *reinterpret_cast<uint2*>(a.hxn + xfrag_off(jb, n0, steps_n)) =
              make_uint2(pack_bf2(o0 * gn.x, o1 * gn.y), pack_bf2(o2 * gn.z, o3 * gn.w));
        }
        s2 = o0 * o0 + o1 * o1 + o2 * o2 + o3 * o3;
      }
      // this tile's share of sum x1^2 per batch row (whole wave: shuffles)
      s2 += __shfl_xor(s2, 16, 64);
      s2 += __shfl_xor(s2, 32, 64);
      if (active && g == 0 && a.ssq_out && n0 < a.n_rows) a.ssq_out[(size_t)jb * a.ssq_np + (n0 >> 4)] = s2;
    } else if (MODE == MODE_GATEUP) {
      const int n0 = tile_row0(0, r) + 4 * g;
      if (active && n0 < a.n_rows) {
        float m[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float ga = v[0][e] * rho, up = v[TW - 1][e] * rho;
          m[e] = ga / (1.f + __expf(-ga)) * up;
        }
        *reinterpret_cast<uint2*>(a.mbuf + xfrag_off(jb, n0, steps_n)) = make_uint2(pack_bf2(m[0], m[1]), pack_bf2(m[2], m[3]));
      }
    } else {  // MODE_LM
      if (active) {
#pragma unroll
        for (int t = 0; t < TW; ++t) {
          const int n0 = tile_row0(t, r) + 4 * g;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n0 + e < a.n_rows) a.logits[(size_t)jb * a.n_rows + n0 + e] = v[t][e] * rho;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One-time pre-shuffle of a [N][K] weight matrix into fragment order: tile (rt, s) of 16 rows x
// 32 k is 64 lanes x 8 elements, lane = row%16 + 16*((k%32)/8); rows >= N and k >= K are zero.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_pack_weight(const unsigned short* src, unsigned short* dst, int N, int K,
                                                     int steps, long long n_frag) {
  const long long f = (long long)blockIdx.x * 256 + threadIdx.x;
  if (f >= n_frag) return;
  const int lane = (int)(f & 63);
  const long long tile = f >> 6;
  const int s = (int)(tile % steps), rt = (int)(tile / steps);
  const int n = rt * 16 + (lane & 15), k = s * 32 + (lane >> 4) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (n < N && k < K) v = *reinterpret_cast<const uint4*>(src + (size_t)n * K + k);  // K % 8 == 0
  *reinterpret_cast<uint4*>(dst + f * 8) = v;
}

// ---------------------------------------------------------------------------------------------
// Step preparation: operand and sum of squares of the first layer, rotary table, cleared
// accumulators.  One workgroup per sequence; loads are issued in groups of four 16-byte words
// so that the kernel costs a couple of memory round trips, not one per element.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_decode_prep(int H, int d, int n_ssq, int bpad, int ssq_np, const int* token_ids,
                                                     const unsigned short* emb, int vocab, const float* x_in, float* xa,
                                                     const float* g1, unsigned short* hx1, float* ssq, float* rope,
                                                     const int* kv_len, const double* inv_freq, int* err_flag) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int steps = (H + 31) >> 5;
  float s2 = 0.f;
  int tok = 0;
  if (token_ids) {
    tok = token_ids[b];
    if (tok < 0 || tok >= vocab) {
      if (tid == 0) atomicOr(err_flag, 2);
      tok = 0;
    }
  }
  const int n4 = H >> 2;  // H % 8 == 0
#pragma unroll 4
  for (int k4 = tid; k4 < n4; k4 += 256) {
    float4 v;
    if (token_ids) {
      const uint2 e = *reinterpret_cast<const uint2*>(emb + (size_t)tok * H + k4 * 4);
      v = make_float4(__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xffff0000u), __uint_as_float(e.y << 16),
                      __uint_as_float(e.y & 0xffff0000u));
      *reinterpret_cast<float4*>(xa + (size_t)b * H + k4 * 4) = v;
    } else {
      v = *reinterpret_cast<const float4*>(x_in + (size_t)b * H + k4 * 4);
    }
    const float4 gg = *reinterpret_cast<const float4*>(g1 + k4 * 4);
    *reinterpret_cast<uint2*>(hx1 + xfrag_off(b, k4 * 4, steps)) =
        make_uint2(pack_bf2(v.x * gg.x, v.y * gg.y), pack_bf2(v.z * gg.z, v.w * gg.w));
    s2 += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  __shared__ float sh[4];
  s2 = wave_sum(s2);
  if ((tid & 63) == 0) sh[tid >> 6] = s2;
  __syncthreads();
  // slot 0 of this row: the whole sum in entry 0, zeros in the others; and in every later slot the padding entries past
  // the tiles their producers write (the consumers add all ssq_np entries of a row)
  const int n_tiles = (H + 15) >> 4;
  for (int i = tid; i < ssq_np; i += 256) ssq[(size_t)b * ssq_np + i] = i == 0 ? (sh[0] + sh[1]) + (sh[2] + sh[3]) : 0.f;
  for (int i = tid; i < (n_ssq - 1) * (ssq_np - n_tiles); i += 256) {
    const int slot = 1 + i / (ssq_np - n_tiles), e = n_tiles + i % (ssq_np - n_tiles);
    ssq[((size_t)slot * bpad + b) * ssq_np + e] = 0.f;
  }
  const int half = d >> 1;
  const double pos = (double)kv_len[b];
  for (int i = tid; i < half; i += 256) {
    // angle = pos * base^(-2i/d) in double, reduced to [-pi, pi] before the fp32 sin/cos
    const double ang = pos * inv_freq[i];
    const double red = ang - 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
    float sn, cs;
    sincosf((float)red, &sn, &cs);
    rope[((size_t)b * half + i) * 2 + 0] = cs;
    rope[((size_t)b * half + i) * 2 + 1] = sn;
  }
}

// ---------------------------------------------------------------------------------------------
// Paged attention for one new token per sequence (the bs*seqlen term of the paper's Eq. 1).
// Workgroup = (chunk of CH tokens, KV head, sequence); each of the 4 waves takes CH/64 pages of
// 16 tokens, issues all its K and V loads up front (16 B per lane; a page of one head is 4 KiB
// contiguous, a wave instruction reads 1 KiB of it), takes the dot products on the vector ALUs
// with wavefront shuffles, and the workgroup merges its waves in LDS.  With more than one chunk
// in the grid every workgroup writes a (max, sum, unnormalised output) partial that
// k_attn_merge combines.
// ---------------------------------------------------------------------------------------------
// Sum over the LPT (8 or 16) lanes that share a token, the same bits in every one of them.  The exchanges are DPP
// operands of the adds (mirror of the 16-lane row, mirror of its 8-lane halves, then inside quads): the cross-lane
// network of the vector ALU, not LDS -- with wavefront shuffles (ds_bpermute) the four query heads of a grouped-query
// chunk kept the LDS pipe busier than the K/V stream kept HBM.  Every step adds the two values of a pair in both
// lanes of the pair, so all lanes end with identical sums.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
template <int LPT>
__device__ __forceinline__ float token_lanes_sum(float s) {
  static_assert(LPT == 8 || LPT == 16, "a token's head vector spans 8 or 16 lanes");
  if (LPT == 16) s += dpp_f<0x140>(s);  // lane i with 15 - i
  s += dpp_f<0x141>(s);                 // lane i with 7 - i of its half row
  s += dpp_f<0x4E>(s);                  // i with i ^ 2
  s += dpp_f<0xB1>(s);                  // i with i ^ 1
  return s;
}

// Waves per SIMD the register allocation aims at.  What the K/V stream reaches follows the bytes in flight per compute
// unit (a workgroup keeps all of its CH tokens in flight): four query heads per KV head at d = 128 need 131 registers
// left alone, three short of a fourth wave per SIMD, that is of 256 instead of 192 KiB in flight.
template <int D, int G>
constexpr int attn_min_waves() { return (D == 128 && G == 4) ? 4 : 1; }

template <int D, int G, int CH>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(attn_min_waves<D, G>(), 8))) k_paged_attn(const float* qbuf, const int* kv_len, const int* page_table,
                                                    int max_pages, int layer, int n_q, int n_kv, const char* slab,
                                                    KvGeom geom, float* part, int max_chunks, unsigned short* obuf,
                                                    int* err_flag) {
  constexpr int LPT = D / 8;         // lanes per token
  constexpr int TPI = 64 / LPT;      // tokens per load instruction
  constexpr int IT = kPageTokens / TPI;
  constexpr int PW = CH / kPageTokens / 4;  // pages per wave
  const int b = blockIdx.z, c = blockIdx.y, ch = blockIdx.x;
  const int n_tot = kv_len[b] + 1;
  // the grid covers the caller's bound max_kv_len: a longer sequence would lose its newest tokens without a word
  if (ch == 0 && c == 0 && threadIdx.x == 0 && (n_tot > (int)gridDim.x * CH || n_tot > max_pages * kPageTokens))
    atomicOr(err_flag, 4);
  if (ch * CH >= n_tot) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int dg = lane % LPT, tl = lane / LPT;
  const int QD = n_q * D;

  // Every load below is unconditional so that all of them are in flight together: page ids
  // past the end of the sequence are replaced by the sequence's last page (valid memory), and
  // what they return is discarded by the `ok` masks.
  uint4 kf[PW][IT], vf[PW][IT];
  bool ok[PW][IT];
  int pg[PW];
  const int last_lp = min((n_tot - 1) / kPageTokens, max_pages - 1);
#pragma unroll
  for (int pp = 0; pp < PW; ++pp) {
    const int lp = ch * (CH / kPageTokens) + wave * PW + pp;
    pg[pp] = page_table[(size_t)b * max_pages + min(lp, last_lp)];
  }
#pragma unroll
  for (int pp = 0; pp < PW; ++pp) {
    const int lp = ch * (CH / kPageTokens) + wave * PW + pp;
    const int tb = lp * kPageTokens;
    bool pgok = lp <= last_lp;
    if (pg[pp] < 0 || pg[pp] >= geom.n_pages_total) {
      if (pgok && lane == 0) atomicOr(err_flag, 1);
      pg[pp] = 0;
      pgok = false;
    }
    const size_t offk = kv_page_off(geom, pg[pp], layer, 0);
    const size_t offv = kv_page_off(geom, pg[pp], layer, 1);
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int slot = it * TPI + tl;
      ok[pp][it] = pgok && (tb + slot) < n_tot;
      const size_t eo = ((size_t)(c * kPageTokens + slot) * D + dg * 8) * sizeof(unsigned short);
      kf[pp][it] = *reinterpret_cast<const uint4*>(slab + offk + eo);
      vf[pp][it] = *reinterpret_cast<const uint4*>(slab + offv + eo);
    }
  }
#pragma unroll
  for (int pp = 0; pp < PW; ++pp)
#pragma unroll
    for (int it = 0; it < IT; ++it)
      if (!ok[pp][it]) kf[pp][it] = vf[pp][it] = make_uint4(0, 0, 0, 0);

  // scores in the log2 domain: s = q.k / sqrt(D) * log2(e)
  const float scale = 1.4426950408889634f * rsqrtf((float)D);
  float qv[G][8];
#pragma unroll
  for (int gq = 0; gq < G; ++gq) {
    const float* q = qbuf + (size_t)b * QD + (c * G + gq) * D + dg * 8;
    const float4 q0 = *reinterpret_cast<const float4*>(q), q1 = *reinterpret_cast<const float4*>(q + 4);
    qv[gq][0] = q0.x * scale; qv[gq][1] = q0.y * scale; qv[gq][2] = q0.z * scale; qv[gq][3] = q0.w * scale;
    qv[gq][4] = q1.x * scale; qv[gq][5] = q1.y * scale; qv[gq][6] = q1.z * scale; qv[gq][7] = q1.w * scale;
  }

  float sc[G][PW][IT];
  float mw[G];
#pragma unroll
  for (int gq = 0; gq < G; ++gq) mw[gq] = -INFINITY;
#pragma unroll
  for (int pp = 0; pp < PW; ++pp)
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      float kk[8];
      unpack8(kf[pp][it], kk);
#pragma unroll
      for (int gq = 0; gq < G; ++gq) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += qv[gq][e] * kk[e];
        s = token_lanes_sum<LPT>(s);
        s = ok[pp][it] ? s : -INFINITY;
        sc[gq][pp][it] = s;
        mw[gq] = fmaxf(mw[gq], s);
      }
    }
  float lw[G], acc[G][8];
#pragma unroll
  for (int gq = 0; gq < G; ++gq) {
#pragma unroll
    for (int o = LPT; o < 64; o <<= 1) mw[gq] = fmaxf(mw[gq], __shfl_xor(mw[gq], o, 64));
    lw[gq] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[gq][e] = 0.f;
  }
#pragma unroll
  for (int pp = 0; pp < PW; ++pp)
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      float vv[8];
      unpack8(vf[pp][it], vv);
#pragma unroll
      for (int gq = 0; gq < G; ++gq) {
        // the hardware exponential as it is: the argument is <= 0 and a result below the normal range may go to zero
        // (the library call rescales around the instruction to return subnormals)
        const float p = ok[pp][it] ? __builtin_amdgcn_exp2f(sc[gq][pp][it] - mw[gq]) : 0.f;
        lw[gq] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[gq][e] += p * vv[e];
      }
    }
#pragma unroll
  for (int gq = 0; gq < G; ++gq) {
#pragma unroll
    for (int o = LPT; o < 64; o <<= 1) {
      lw[gq] += __shfl_xor(lw[gq], o, 64);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[gq][e] += __shfl_xor(acc[gq][e], o, 64);
    }
  }

  __shared__ float s_m[4][G], s_l[4][G], s_o[4][G][D];
  if (tl == 0) {
#pragma unroll
    for (int gq = 0; gq < G; ++gq) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_o[wave][gq][dg * 8 + e] = acc[gq][e];
      if (dg == 0) {
        s_m[wave][gq] = mw[gq];
        s_l[wave][gq] = lw[gq];
      }
    }
  }
  __syncthreads();
  const int steps_o = (QD + 31) >> 5;
  for (int idx = tid; idx < G * D; idx += 256) {
    const int gq = idx / D, e = idx - gq * D;
    const float M = fmaxf(fmaxf(s_m[0][gq], s_m[1][gq]), fmaxf(s_m[2][gq], s_m[3][gq]));
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = (s_m[w][gq] == -INFINITY) ? 0.f : exp2f(s_m[w][gq] - M);
      L += s_l[w][gq] * f;
      o += s_o[w][gq][e] * f;
    }
    const int head = c * G + gq;
    if (gridDim.x == 1) {
      obuf[xfrag_off(b, head * D + e, steps_o)] = f2bf(o / L);
    } else {
      float* p = part + (((size_t)b * n_q + head) * max_chunks + ch) * (D + 2);
      p[2 + e] = o;
      if (e == 0) {
        p[0] = M;
        p[1] = L;
      }
    }
  }
}

// Merge of the per-chunk partials: one workgroup per (query head, sequence).  A separate launch
// rather than a last-arriver merge inside the attention kernel: a device-scope fence per
// workgroup writes back and invalidates the whole L2 of its XCD on this chip and was measured
// at ten times the cost of the attention itself.
template <int D, int CH>
__global__ void __launch_bounds__(D) k_attn_merge(const float* part, const int* kv_len, int n_q, int max_chunks,
                                                  unsigned short* obuf) {
  const int head = blockIdx.x, b = blockIdx.y, e = threadIdx.x;
  const int n_tot = kv_len[b] + 1;
  const int nch = min((n_tot + CH - 1) / CH, max_chunks);
  if (nch < 1) return;
  const float* p = part + (((size_t)b * n_q + head) * max_chunks) * (D + 2);
  float M = -INFINITY, L = 0.f, o = 0.f;
  for (int i0 = 0; i0 < nch; i0 += 8) {  // eight chunks per round trip
    float m[8], l[8], v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float* pi = p + (size_t)min(i0 + u, nch - 1) * (D + 2);
      m[u] = pi[0];
      l[u] = pi[1];
      v[u] = pi[2 + e];
    }
    float Mn = M;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + u < nch) Mn = fmaxf(Mn, m[u]);
    const float f0 = (M == -INFINITY) ? 0.f : exp2f(M - Mn);
    L *= f0;
    o *= f0;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + u < nch) {
        const float f = exp2f(m[u] - Mn);
        L += l[u] * f;
        o += v[u] * f;
      }
    M = Mn;
  }
  obuf[xfrag_off(b, head * D + e, (n_q * D + 31) >> 5)] = f2bf(o / L);
}

// argmax over the vocabulary in two launches: kArgSeg workgroups per sequence each find the first maximum of
// their slice, one wave per sequence then picks among the slices (a single workgroup per sequence took 0.2 ms on
// a 128k vocabulary whatever the batch).  Ties go to the smaller index at both levels: the first maximum, as in the
// plain definition.
constexpr int kArgSeg = 64;

__device__ __forceinline__ bool arg_better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ void __launch_bounds__(256) k_argmax_part(const float* logits, int V, float* part_v, int* part_i) {
  const int seg = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int len = (V + kArgSeg - 1) / kArgSeg;
  const int lo = seg * len, hi = min(V, lo + len);
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = lo + tid; i < hi; i += 256) {
    const float v = logits[(size_t)b * V + i];
    if (v > best) {  // indices increase per thread: the first maximum is kept
      best = v;
      bi = i;
    }
  }
  for (int o = 1; o < 64; o <<= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (arg_better(ov, oi, best, bi)) {
      best = ov;
      bi = oi;
    }
  }
  __shared__ float sv[4];
  __shared__ int si[4];
  if ((tid & 63) == 0) {
    sv[tid >> 6] = best;
    si[tid >> 6] = bi;
  }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w)
      if (arg_better(sv[w], si[w], best, bi)) {
        best = sv[w];
        bi = si[w];
      }
    part_v[b * kArgSeg + seg] = best;
    part_i[b * kArgSeg + seg] = bi;
  }
}

__global__ void __launch_bounds__(64) k_argmax_final(const float* part_v, const int* part_i, int* next_token) {
  const int b = blockIdx.x, lane = threadIdx.x;
  static_assert(kArgSeg == 64, "one lane per slice");
  float best = part_v[b * kArgSeg + lane];
  int bi = part_i[b * kArgSeg + lane];
  for (int o = 1; o < 64; o <<= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (arg_better(ov, oi, best, bi)) {
      best = ov;
      bi = oi;
    }
  }
  if (lane == 0) next_token[b] = bi;
}

template <int MODE, int NB, int TW, int KW, int U, int RT>
void launch_skinny(const SkinnyArgs& a, int n_wg, hipStream_t st) {
  // dynamic LDS: the staged partial sums of squares of NB x 16 batch rows (small batches of the normalised GEMMs)
  const size_t lds = (MODE != MODE_RESID && NB <= 2) ? (size_t)NB * 16 * (((size_t)a.ssq_np * 4 + 1023) & ~size_t(1023)) : 0;
  hipLaunchKernelGGL((k_skinny<MODE, NB, TW, KW, U, RT>), dim3((n_wg + RT - 1) / RT), dim3(TW * KW * 64), lds, st, a);
}

// passes of at most 64 batch rows (128 where the workgroup has eight waves to finish eight batch tiles and more than
// 64 rows are left: every pass streams the whole weight matrix again); NB = 16-row batch tiles per pass.
// n_wg: workgroups at one weight tile per wave.
template <int MODE, int TW, int KW>
void dispatch_skinny(SkinnyArgs a, int n_wg, hipStream_t st) {
  // Two weight tiles per wave (RT = 2) halve the workgroups.  Measured on 256 compute units: with 64 rows per pass
  // it pays only where two workgroups per compute unit remain (gate/up, output layer; the 256-tile projections lost
  // more from running on half the chip than they gained); with 128 rows per pass it pays everywhere.  q,k,v: the
  // rotation indices of a head (d/2) split into groups of 16 * RT; d = 32 has a single 16-row group.
  const bool rt_ok = MODE != MODE_QKV || (a.d >> 5) % 2 == 0;
  const bool rt2_64 = rt_ok && n_wg >= 2 * kComputeUnits;
  for (int b0 = 0; b0 < a.B;) {
    a.b0 = b0;
    const int left = a.B - b0;
    if constexpr (TW * KW >= 8) {
      if (left > 64) {
        if (rt_ok)
          launch_skinny<MODE, 8, TW, KW, 1, 2>(a, n_wg, st);
        else
          launch_skinny<MODE, 8, TW, KW, 1, 1>(a, n_wg, st);
        b0 += 128;
        continue;
      }
    }
    const int nb = (min(left, 64) + 15) / 16;
    if (nb == 1)
      launch_skinny<MODE, 1, TW, KW, 8, 1>(a, n_wg, st);
    else if (nb == 2)
      launch_skinny<MODE, 2, TW, KW, 4, 1>(a, n_wg, st);
    else if (rt2_64)
      launch_skinny<MODE, 4, TW, KW, 2, 2>(a, n_wg, st);
    else
      launch_skinny<MODE, 4, TW, KW, 2, 1>(a, n_wg, st);
    b0 += 64;
  }
}

template <int D, int G, int CH>
void launch_attn(harli_ctx* c, const DecodeWs& w, const harli_decode_batch* b, int layer, hipStream_t st) {
  const harli_model_cfg& m = c->cfg;
  const int n_chunks = (b->max_kv_len + CH - 1) / CH;
  hipLaunchKernelGGL((k_paged_attn<D, G, CH>), dim3(n_chunks, m.n_kv_heads, b->batch), dim3(256), 0, st, w.qbuf,
                     b->kv_len, b->page_table, b->max_pages, layer, m.n_q_heads, m.n_kv_heads, c->slab, c->geom,
                     w.att_part, w.max_chunks, static_cast<unsigned short*>(w.obuf), w.err_flag);
  if (n_chunks > 1)
    hipLaunchKernelGGL((k_attn_merge<D, CH>), dim3(m.n_q_heads, b->batch), dim3(D), 0, st, w.att_part, b->kv_len,
                       m.n_q_heads, w.max_chunks, static_cast<unsigned short*>(w.obuf));
}

}  // namespace

namespace harli {

harli_status decode_step_f32(harli_ctx* c, const harli_decode_batch* b, hipStream_t st);  // decode_generic.hip

size_t packed_weight_elems(int N, int K) { return (size_t)((N + 15) / 16) * ((K + 31) / 32) * 512; }

// dst must hold packed_weight_elems(N, K) bf16; rows [row_tile0*16, ...) of the packed matrix are written
harli_status pack_weight(const void* src, void* dst, int N, int K, int row_tile0, hipStream_t st) {
  const int steps = (K + 31) / 32;
  const long long n_frag = (long long)((N + 15) / 16) * steps * 64;
  unsigned short* d = static_cast<unsigned short*>(dst) + (size_t)row_tile0 * steps * 512;
  hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)((n_frag + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned short*>(src), d, N, K, steps, n_frag);
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

}  // namespace harli

namespace {

// Argument checks shared by the two entry points (host only; nothing is enqueued on failure).
harli_status check_decode_args(harli_ctx* c, const harli_decode_batch* b) {
  if (!c || !b) return fail(HARLI_ERR_INVALID, "decode_step: null argument");
  const harli_model_cfg& m = c->cfg;
  if (b->batch < 1 || b->batch > m.max_batch)
    return fail(HARLI_ERR_INVALID, "decode_step: batch %d outside 1..%d", b->batch, m.max_batch);
  if (!b->kv_len || !b->page_table) return fail(HARLI_ERR_INVALID, "decode_step: kv_len and page_table are required");
  if (!b->token_ids && !b->x_in) return fail(HARLI_ERR_INVALID, "decode_step: give token_ids or x_in");
  if (b->token_ids && !c->emb) return fail(HARLI_ERR_INVALID, "decode_step: token_ids need an embedding table");
  if ((b->logits || b->next_token) && (!c->w_lm || !c->g_final))
    return fail(HARLI_ERR_INVALID, "decode_step: logits need g_final and w_lm");
  if (b->next_token && !b->logits) return fail(HARLI_ERR_INVALID, "decode_step: next_token needs a logits buffer");
  if (b->max_kv_len < 1 || b->max_kv_len > m.max_seq_len)
    return fail(HARLI_ERR_INVALID, "decode_step: max_kv_len %d outside 1..%d", b->max_kv_len, m.max_seq_len);
  if ((long long)b->max_pages * c->geom.page_tokens < b->max_kv_len)
    return fail(HARLI_ERR_INVALID, "decode_step: page table rows of %d pages cannot hold %d tokens", b->max_pages,
                b->max_kv_len);
  return HARLI_OK;
}

// The step on bf16 storage; every intermediate buffer comes from `w`.
harli_status decode_step_bf16(harli_ctx* c, const harli_decode_batch* b, hipStream_t st, const DecodeWs& w) {
  const harli_model_cfg& m = c->cfg;
  const int B = b->batch, H = m.hidden, d = m.head_dim, QD = m.n_q_heads * d, F = m.ffn, L = m.n_layers;
  const int n_ssq = 2 * L + 1;
  const int np = ssq_entries(H);
  hipLaunchKernelGGL(k_decode_prep, dim3(B), dim3(256), 0, st, H, d, n_ssq, w.bpad, np, b->token_ids,
                     static_cast<const unsigned short*>(c->emb), m.vocab, b->x_in, w.xa, c->layers[0].g1,
                     static_cast<unsigned short*>(w.hx1), w.ssq, w.rope, b->kv_len, w.inv_freq, w.err_flag);

  const float* xcur = b->token_ids ? w.xa : b->x_in;
  float* ping[2] = {w.xb, w.xa};  // layer l writes ping[l&1]; layer 0 must not overwrite xa (it can be its input)
  const int G = m.n_q_heads / m.n_kv_heads;
  // above 32 sequences the layer GEMMs run as tiled MFMA GEMMs with their epilogues in a second kernel (decode_large.h);
  // a caller's buffer without the workspace for their partial tiles keeps every batch on the small-batch kernels
  const bool large = B >= dg_min_batch() && w.part != nullptr;
  int n_cu = cu_stream_count(st);  // a stream confined to a share of the compute units (Sec. 6.2)
  if (n_cu < 1) n_cu = c->n_cu;
  const int x_tiles = w.bpad / 16;

  for (int l = 0; l < L; ++l) {
    const LayerDev& lw = c->layers[l];
    SkinnyArgs a{};
    a.B = B;
    a.eps = m.rms_eps;
    a.inv_dim = 1.f / (float)H;
    a.err_flag = w.err_flag;
    // --- QKV + rotary + append
    a.x = static_cast<const unsigned short*>(w.hx1);
    a.K = H;
    a.n_rows = QD;
    a.w0 = static_cast<const unsigned short*>(lw.wp[0]);
    a.ssq_np = np;
    a.ssq_in = w.ssq + (size_t)(2 * l) * w.bpad * np;
    a.qbuf = w.qbuf;
    a.rope = w.rope;
    a.kv_len = b->kv_len;
    a.page_table = b->page_table;
    a.max_pages = b->max_pages;
    a.layer = l;
    a.n_q = m.n_q_heads;
    a.n_kv = m.n_kv_heads;
    a.d = d;
    a.slab = c->slab;
    a.geom = c->geom;
    for (int t = 0; t < 3; ++t) a.bias[t] = lw.bias[t];
    if (large) {
      harli_status rc = dg_launch(DG_QKV, a, x_tiles, w.part, w.part_bytes, n_cu, st);
      if (rc != HARLI_OK) return rc;
    } else {
      dispatch_skinny<MODE_QKV, 2, 2>(a, (m.n_q_heads + 2 * m.n_kv_heads) * (d / 32), st);
    }
    // --- attention
    if (d == 128 && G == 1) launch_attn<128, 1, 256>(c, w, b, l, st);
    else if (d == 128 && G == 2) launch_attn<128, 2, 256>(c, w, b, l, st);
    else if (d == 128 && G == 4) launch_attn<128, 4, 128>(c, w, b, l, st);
    else if (d == 128 && G == 8) launch_attn<128, 8, 128>(c, w, b, l, st);
    else if (d == 128 && G == 3) launch_attn<128, 3, 128>(c, w, b, l, st);
    else if (d == 128 && G == 5) launch_attn<128, 5, 128>(c, w, b, l, st);
    else if (d == 128 && G == 6) launch_attn<128, 6, 128>(c, w, b, l, st);
    else if (d == 128 && G == 7) launch_attn<128, 7, 128>(c, w, b, l, st);
    else if (d == 64 && G == 1) launch_attn<64, 1, 256>(c, w, b, l, st);
    else if (d == 64 && G == 2) launch_attn<64, 2, 256>(c, w, b, l, st);
    else if (d == 64 && G == 4) launch_attn<64, 4, 256>(c, w, b, l, st);
    else return fail(HARLI_ERR_INVALID, "decode_step: head_dim %d with group %d is not supported", d, G);
    // --- output projection + residual, operand of the FFN
    a.x = static_cast<const unsigned short*>(w.obuf);
    a.K = QD;
    a.n_rows = H;
    a.w0 = static_cast<const unsigned short*>(lw.wp[3]);
    a.res = xcur;
    a.out = w.x1;
    a.gnext = lw.g2;
    a.hxn = static_cast<unsigned short*>(w.hx2);
    a.ssq_out = w.ssq + (size_t)(2 * l + 1) * w.bpad * np;
    if (large) {
      harli_status rc = dg_launch(DG_RESID, a, x_tiles, w.part, w.part_bytes, n_cu, st);
      if (rc != HARLI_OK) return rc;
    } else {
      dispatch_skinny<MODE_RESID, 1, 8>(a, (H + 15) / 16, st);
    }
    // --- gate/up + SwiGLU
    a.x = static_cast<const unsigned short*>(w.hx2);
    a.K = H;
    a.n_rows = F;
    a.w0 = static_cast<const unsigned short*>(lw.wp[4]);
    a.w1 = static_cast<const unsigned short*>(lw.wp[5]);
    a.ssq_in = w.ssq + (size_t)(2 * l + 1) * w.bpad * np;
    a.mbuf = static_cast<unsigned short*>(w.mbuf);
    if (large) {
      harli_status rc = dg_launch(DG_GATEUP, a, x_tiles, w.part, w.part_bytes, n_cu, st);
      if (rc != HARLI_OK) return rc;
    } else {
      dispatch_skinny<MODE_GATEUP, 2, 4>(a, (F + 15) / 16, st);
    }
    // --- down projection + residual, operand of the next layer (or of the output layer)
    const bool last = (l == L - 1);
    float* xnext = (last && b->x_out) ? b->x_out : ping[l & 1];
    a.x = static_cast<const unsigned short*>(w.mbuf);
    a.K = F;
    a.n_rows = H;
    a.w0 = static_cast<const unsigned short*>(lw.wp[6]);
    a.res = w.x1;
    a.out = xnext;
    a.gnext = last ? c->g_final : c->layers[l + 1].g1;
    a.hxn = (last && !b->logits) ? nullptr : static_cast<unsigned short*>(w.hx1);
    a.ssq_out = w.ssq + (size_t)(2 * l + 2) * w.bpad * np;
    if (large) {
      harli_status rc = dg_launch(DG_RESID, a, x_tiles, w.part, w.part_bytes, n_cu, st);
      if (rc != HARLI_OK) return rc;
    } else {
      dispatch_skinny<MODE_RESID, 1, 8>(a, (H + 15) / 16, st);
    }
    xcur = xnext;
  }
  if (b->logits) {
    SkinnyArgs a{};
    a.B = B;
    a.eps = m.rms_eps;
    a.inv_dim = 1.f / (float)H;
    a.x = static_cast<const unsigned short*>(w.hx1);
    a.K = H;
    a.n_rows = m.vocab;
    a.w0 = static_cast<const unsigned short*>(c->wlm_p);
    a.ssq_np = np;
    a.ssq_in = w.ssq + (size_t)(2 * L) * w.bpad * np;
    a.logits = b->logits;
    // the output layer through the tiled path too, when one partial matrix of [batch, vocabulary] fits the workspace
    if (large && dg_plan(B, m.vocab, 1, H, n_cu, w.part_bytes).ksplit >= 1 && (long long)((m.vocab + 15) / 16 + 16) * ((H + 31) / 32) * 1024 < (1ll << 31)) {
      harli_status rc = dg_launch(DG_LM, a, x_tiles, w.part, w.part_bytes, n_cu, st);
      if (rc != HARLI_OK) return rc;
    } else {
      dispatch_skinny<MODE_LM, 2, 4>(a, (m.vocab + 31) / 32, st);
    }
    if (b->next_token) {
      hipLaunchKernelGGL(k_argmax_part, dim3(kArgSeg, B), dim3(256), 0, st, b->logits, m.vocab, w.amax_v, w.amax_i);
      hipLaunchKernelGGL(k_argmax_final, dim3(B), dim3(64), 0, st, w.amax_v, w.amax_i, b->next_token);
    }
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

// ---------------------------------------------------------------------------------------------
// Static scratch of harli_decode_step_static: the step's intermediate buffers for callers that may not allocate.
// One copy of the array exists on every device the library is loaded on, at that device's own address; host code
// never uses the array's name as an address, only the pointer hipGetSymbolAddress returned for the device.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = HARLI_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// device address of `scratch` on the current device (looked up once per device)
harli_status static_scratch(unsigned char** out) {
  int dev = -1;
  HARLI_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(HARLI_ERR_INVALID, "decode_step_static: device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HARLI_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(HARLI_ERR_HIP, "decode_step_static: the scratch symbol has no address on device %d", dev);
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
  return HARLI_OK;
}

// 16-byte fill (a kernel rather than a memset call, so that the step stays capturable in a HIP graph)
__global__ void __launch_bounds__(256) k_zero16(uint4* p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace

extern "C" harli_status harli_decode_step(harli_ctx* c, const harli_decode_batch* b, void* hip_stream) {
  harli_status s = check_decode_args(c, b);
  if (s != HARLI_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (c->cfg.dtype == HARLI_F32) return decode_step_f32(c, b, st);
  return decode_step_bf16(c, b, st, c->dw);
}

extern "C" int32_t harli_decode_tiled_min_batch(void) { return dg_min_batch(); }

extern "C" size_t harli_decode_step_static_bytes(const harli_ctx* c, int32_t batch, int32_t max_kv_len) {
  if (!c || batch < 1 || max_kv_len < 1) return 0;
  const harli_model_cfg& m = c->cfg;
  auto al = [](size_t n) { return (n + 255) & ~size_t(255); };
  auto r32 = [](size_t n) { return (n + 31) & ~size_t(31); };
  const size_t bp = (size_t)(batch + 15) / 16 * 16, H = m.hidden, QD = (size_t)m.n_q_heads * m.head_dim, F = m.ffn;
  const size_t chunks = ((size_t)max_kv_len + 127) / 128;
  size_t n = al(bp * r32(H) * 2) * 2 + al(bp * r32(QD) * 2) + al(bp * r32(F) * 2);       // GEMM operands
  n += al(bp * QD * 4) + 3 * al(bp * H * 4);                                             // q, x1, xa, xb
  n += al(bp * (2 * (size_t)m.n_layers + 1) * ssq_entries(m.hidden) * 4) + al(bp * m.head_dim * 4);  // row norms, rotary table
  n += al(bp * m.n_q_heads * chunks * ((size_t)m.head_dim + 2) * 4);                     // attention partials
  n += 2 * al(bp * 64 * 4);                                                              // argmax partials
  return n;
}

extern "C" harli_status harli_decode_step_static(harli_ctx* c, const harli_decode_batch* b, void* hip_stream) {
  harli_status s = check_decode_args(c, b);
  if (s != HARLI_OK) return s;
  const harli_model_cfg& m = c->cfg;
  if (m.dtype != HARLI_BF16) return fail(HARLI_ERR_INVALID, "decode_step_static: bf16 storage only");
  const size_t need = harli_decode_step_static_bytes(c, b->batch, b->max_kv_len);
  if (need > kStaticScratchBytes)
    return fail(HARLI_ERR_INVALID, "decode_step_static: batch %d with max_kv_len %d needs %zu bytes of scratch, the static buffer holds %zu",
                b->batch, b->max_kv_len, need, kStaticScratchBytes);
  unsigned char* base = nullptr;
  s = static_scratch(&base);
  if (s != HARLI_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the same layout harli_decode_step_static_bytes adds up, sized by this call's batch and length bound
  auto al = [](size_t n) { return (n + 255) & ~size_t(255); };
  auto r32 = [](size_t n) { return (n + 31) & ~size_t(31); };
  const size_t bp = (size_t)(b->batch + 15) / 16 * 16, H = m.hidden, QD = (size_t)m.n_q_heads * m.head_dim, F = m.ffn;
  const size_t chunks = ((size_t)b->max_kv_len + 127) / 128;
  size_t off = 0;
  auto take = [&](size_t n) {
    unsigned char* p = base + off;
    off += al(n);
    return p;
  };
  DecodeWs w;
  w.bpad = (int)bp;
  w.max_chunks = (int)chunks;
  w.hx1 = take(bp * r32(H) * 2);
  w.hx2 = take(bp * r32(H) * 2);
  w.obuf = take(bp * r32(QD) * 2);
  w.mbuf = take(bp * r32(F) * 2);
  const size_t operand_bytes = off;
  w.qbuf = reinterpret_cast<float*>(take(bp * QD * 4));
  w.x1 = reinterpret_cast<float*>(take(bp * H * 4));
  w.xa = reinterpret_cast<float*>(take(bp * H * 4));
  w.xb = reinterpret_cast<float*>(take(bp * H * 4));
  w.ssq = reinterpret_cast<float*>(take(bp * (2 * (size_t)m.n_layers + 1) * ssq_entries(m.hidden) * 4));
  w.rope = reinterpret_cast<float*>(take(bp * m.head_dim * 4));
  w.att_part = reinterpret_cast<float*>(take(bp * m.n_q_heads * chunks * ((size_t)m.head_dim + 2) * 4));
  w.amax_v = reinterpret_cast<float*>(take(bp * 64 * 4));
  w.amax_i = reinterpret_cast<int*>(take(bp * 64 * 4));
  w.inv_freq = c->dw.inv_freq;  // constants and the error flag made in harli_ctx_create
  w.err_flag = c->dw.err_flag;
  if (off != need) return fail(HARLI_ERR_STATE, "decode_step_static: layout of %zu bytes against %zu counted", off, need);
  // The array keeps what the last call (of any shape) left.  The GEMM operands must start at zero: contraction
  // positions past K (up to the next multiple of 32) are multiplied with the zero padding of the weights, and stale
  // bits there may read as NaN.  Everything else is written before it is read (the row-norm partials are written by their
  // producers and their padding by the step's first kernel; batch rows past `batch` only reach output columns that are never stored).
  const size_t n16 = operand_bytes / 16;
  hipLaunchKernelGGL(k_zero16, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, reinterpret_cast<uint4*>(base), n16);
  return decode_step_bf16(c, b, st, w);
}
