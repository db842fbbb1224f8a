// Element-wise, reduction and skinny kernels of the LoRA finetune unit (Harli Sec. 2.1: forward,
// backward with adapter gradients only; Sec. 6.1: one transformer layer per call).  These are
// the HBM-bound pieces between the MFMA GEMMs: every kernel reads and writes each element once
// with 8- or 16-byte accesses.
#include "ft_kernels.h"

#include <algorithm>

#include "ft_elem.h"

namespace harli {
namespace {

__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return r;
}

// ---------------------------------------------------------------- RMSNorm
__global__ void __launch_bounds__(256) k_rmsnorm_fwd(const float* x, const float* g, bf* h, float* rho, int H, float eps, int* flag) {
  __shared__ float sh[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  const float* xr = x + (size_t)t * H;
  float s2 = 0.f;
  for (int k = tid * 4; k < H; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    s2 += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  s2 = block_sum_256(s2, sh);
  const float r = rsqrtf(s2 / (float)H + eps);
  if (tid == 0) rho[t] = r;
  bool over = false;
  for (int k = tid * 4; k < H; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    const float4 gg = *reinterpret_cast<const float4*>(g + k);
    *reinterpret_cast<uint2*>(h + (size_t)t * H + k) =
        make_uint2(PACK2G(v.x * r * gg.x, v.y * r * gg.y, over), PACK2G(v.z * r * gg.z, v.w * r * gg.w, over));
  }
  elem_flag(over, flag);
}

__global__ void __launch_bounds__(256) k_rmsnorm_bwd(const float* dh, const float* x, const float* rho, const float* g,
                                                     const float* dres, float* dx, bf* dx16, int H, const float* res_mul,
                                                     const float* out_mul, int* flag) {
  __shared__ float sh[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  const float r = rho[t];
  const float rm = res_mul ? *res_mul : 1.f, om = out_mul ? *out_mul : 1.f;
  const float* xr = x + (size_t)t * H;
  const float* dr = dh + (size_t)t * H;
  float dot = 0.f;
  for (int k = tid * 4; k < H; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    const float4 d = *reinterpret_cast<const float4*>(dr + k);
    const float4 gg = *reinterpret_cast<const float4*>(g + k);
    dot += d.x * gg.x * v.x + d.y * gg.y * v.y + d.z * gg.z * v.z + d.w * gg.w * v.w;
  }
  dot = block_sum_256(dot, sh);
  const float c = dot * r * r / (float)H;  // mean(dh*g*xhat) * rho, with xhat = x * rho
  bool over = false;
  for (int k = tid * 4; k < H; k += 1024) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    const float4 d = *reinterpret_cast<const float4*>(dr + k);
    const float4 gg = *reinterpret_cast<const float4*>(g + k);
    const float4 rs = dres ? *reinterpret_cast<const float4*>(dres + (size_t)t * H + k) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 o;
    o.x = om * (rs.x * rm + r * (d.x * gg.x - v.x * c));
    o.y = om * (rs.y * rm + r * (d.y * gg.y - v.y * c));
    o.z = om * (rs.z * rm + r * (d.z * gg.z - v.z * c));
    o.w = om * (rs.w * rm + r * (d.w * gg.w - v.w * c));
    *reinterpret_cast<float4*>(dx + (size_t)t * H + k) = o;
    if (dx16) *reinterpret_cast<uint2*>(dx16 + (size_t)t * H + k) = make_uint2(PACK2G(o.x, o.y, over), PACK2G(o.z, o.w, over));
  }
  elem_flag(over, flag);
}

// ---------------------------------------------------------------- rotary embedding, pairs (i, i + d/2)
// One workgroup per token.  The d/2 (cos, sin) pairs of the token's position are computed once into LDS (angle
// reduced in double, as the oracle's positions are exact) and shared by every head.  One thread rotates eight
// adjacent pairs with two 16-byte loads and stores when d/2 is a multiple of 8 (rows are 16-byte aligned then:
// heads*d is a multiple of 8); other head sizes take the pair-at-a-time loop.
constexpr int kRopeMaxHalf = 256;
__global__ void __launch_bounds__(256) k_rope(bf* x, int S, int heads, int d, const double* inv_freq, float sign, int* flag) {
  __shared__ float cs_[kRopeMaxHalf], sn_[kRopeMaxHalf];
  const int t = blockIdx.x, half = d >> 1;
  const double pos = (double)(t % S);
  for (int i = threadIdx.x; i < half; i += 256) {
    const double ang = pos * inv_freq[i];
    const double red = ang - 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
    float sn, cs;
    sincosf((float)red, &sn, &cs);
    cs_[i] = cs;
    sn_[i] = sn * sign;
  }
  __syncthreads();
  bf* row = x + (size_t)t * heads * d;
  bool over = false;
  if ((half & 7) == 0) {
    const int per_head = half >> 3;
    for (int idx = threadIdx.x; idx < heads * per_head; idx += 256) {
      const int hh = idx / per_head, i0 = (idx - hh * per_head) * 8;
      bf* p = row + hh * d + i0;
      const uint4 lo4 = *reinterpret_cast<const uint4*>(p), hi4 = *reinterpret_cast<const uint4*>(p + half);
      float lo[8], hi[8], ol[8], oh[8];
      UNPACK8(lo4, lo);
      UNPACK8(hi4, hi);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float cs = cs_[i0 + e], sn = sn_[i0 + e];
        ol[e] = lo[e] * cs - hi[e] * sn;
        oh[e] = hi[e] * cs + lo[e] * sn;
      }
      *reinterpret_cast<uint4*>(p) = make_uint4(PACK2G(ol[0], ol[1], over), PACK2G(ol[2], ol[3], over), PACK2G(ol[4], ol[5], over),
                                                PACK2G(ol[6], ol[7], over));
      *reinterpret_cast<uint4*>(p + half) = make_uint4(PACK2G(oh[0], oh[1], over), PACK2G(oh[2], oh[3], over),
                                                       PACK2G(oh[4], oh[5], over), PACK2G(oh[6], oh[7], over));
    }
    elem_flag(over, flag);
    return;
  }
  for (int idx = threadIdx.x; idx < heads * half; idx += 256) {
    const int hh = idx / half, i = idx - hh * half;
    const float cs = cs_[i], sn = sn_[i];
    bf* p = row + hh * d + i;
    const float lo = E2F(p[0]), hi = E2F(p[half]);
    p[0] = F2EG(lo * cs - hi * sn, over);
    p[half] = F2EG(hi * cs + lo * sn, over);
  }
  elem_flag(over, flag);
}

// ---------------------------------------------------------------- head-wise transposes (64 x 64 tiles through LDS)
// Per sequence b: [S][heads*d] -> [heads*d][S].  Up to three tensors per launch (blockIdx.z = job * Bf + b).  Both
// global sides move 16 bytes per lane (S and heads*d are multiples of 8); the transposition happens in the 2-byte LDS
// writes.
__global__ void __launch_bounds__(256) k_transpose_heads(TransposeJobs jobs, int Bf, int S) {
  __shared__ __align__(16) bf tile[64][72];  // [column][row], rows padded to 144 bytes
  const int job = blockIdx.z / Bf, b = blockIdx.z - job * Bf;
  const int C = jobs.C[job];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  if (c0 >= C) return;
  const bf* src = jobs.in[job] + (long long)b * S * C;
  bf* dst = jobs.out[job] + (long long)b * S * C;
  const int t = threadIdx.x, q8 = (t & 7) * 8, p = t >> 3;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = p + 32 * pass;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r0 + r < S && c0 + q8 < C) v = *reinterpret_cast<const uint4*>(src + (long long)(r0 + r) * C + c0 + q8);
    const unsigned wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[q8 + e][r] = (bf)(wv[e >> 1] >> (16 * (e & 1)));
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int c = p + 32 * pass;
    if (c0 + c < C && r0 + q8 < S)
      *reinterpret_cast<uint4*>(dst + (long long)(c0 + c) * S + r0 + q8) = *reinterpret_cast<const uint4*>(&tile[c][q8]);
  }
}

// ---------------------------------------------------------------- gradient scaling
// The backward pass is linear in dY, so dY is multiplied by a power of two sigma that brings its
// largest magnitude to 2^8 before it is rounded to 16 bits, and 1/sigma is applied where the
// fp32 results leave the unit (dX, dA, dB).  scale[0] = sigma, scale[1] = 1/sigma.
__global__ void __launch_bounds__(256) k_amax(const float* x, long long n4, unsigned* amax_bits) {
  // grid-stride over groups of 1024 float4, four independent 16-byte loads per thread in flight (indices past the
  // end re-read the last element); one atomic per workgroup (same-address atomics serialise)
  __shared__ float wmax[4];
  float m = 0.f;
  for (long long base = (long long)blockIdx.x * 1024 + threadIdx.x; base < n4; base += (long long)gridDim.x * 1024) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = reinterpret_cast<const float4*>(x)[min(base + u * 256, n4 - 1)];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      m = fmaxf(fmaxf(fmaxf(fabsf(v[u].x), fabsf(v[u].y)), fmaxf(fabsf(v[u].z), fabsf(v[u].w))), m);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0)
    atomicMax(amax_bits, __float_as_uint(fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]))));  // non-negative floats order like their bits
}
// sigma from the largest magnitude: the power of two that brings it to 2^target_log2 (1 for an all-zero or non-finite dY)
__device__ __forceinline__ float sigma_of(unsigned amax_bits, int target_log2) {
  const float a = __uint_as_float(amax_bits);
  if (!(a > 0.f && a < INFINITY)) return 1.f;
  int e;
  frexpf(a, &e);  // a = f * 2^e, f in [0.5, 1)
  return ldexpf(1.f, min(max(target_log2 - e, -100), 100));
}
// y = 16-bit(x * sigma).  Every workgroup derives sigma from the maximum that k_amax left in bits[0]; workgroup 0 also
// publishes scale[0] = sigma, scale[1] = 1 / sigma for the kernels downstream and clears bits[1], the slot the next
// call's k_amax will use (the two slots alternate, so no launch is spent on a reset).
__global__ void __launch_bounds__(256) k_f32_to_e_scaled(const float* x, bf* y, long long n4, const unsigned* bits_now,
                                                         unsigned* bits_next, float* scale, int target_log2) {
  const float sg = sigma_of(*bits_now, target_log2);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    scale[0] = sg;
    scale[1] = 1.f / sg;
    *bits_next = 0u;
  }
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const float4 v = reinterpret_cast<const float4*>(x)[i];
  reinterpret_cast<uint2*>(y)[i] = make_uint2(PACK2(v.x * sg, v.y * sg), PACK2(v.z * sg, v.w * sg));
}

// ---------------------------------------------------------------- skinny NT GEMM (LoRA down-projection x.A and dy.B^T)
// Workgroup = 16 rows of X, 8 waves split K, one 16x16x32 MFMA column tile per 16 outputs.  Full 32-wide K steps are
// loaded four at a time, unconditionally; only a last partial step (K % 32) masks its operands.
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;  // native vector: arrays of it stay in registers
__device__ __forceinline__ f32x4 mma16(const u32x4& a, const u32x4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <int NT>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) k_skinny_nt(SkinnyNtJobs jobs, int M, float alpha, int* flag) {
  const SkinnyNtJob& jb = jobs.j[blockIdx.y];
  const bf* X = jb.X;
  const bf* Bm = jb.Bm;
  bf* C = jb.C;
  const long long ldx = jb.ldx, ldb = jb.ldb, ldc = jb.ldc;
  const int N = jb.N, K = jb.K;
  constexpr int NW = 8, U = NT == 1 ? 16 : NT == 2 ? 8 : 4;  // K steps in flight per wave: a wave has few steps, latency is what it waits for
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i16 = lane & 15, g = lane >> 4;
  const int m0 = blockIdx.x * 16;
  const int mr = min(m0 + i16, M - 1);
  const bf* xr = X + (long long)mr * ldx + g * 8;
  const bf* br[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) br[t] = Bm + (long long)min(t * 16 + i16, N - 1) * ldb + g * 8;
  f32x4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int full = K >> 5;  // whole 32-wide steps
  const int s0 = full * wave / NW, s1 = full * (wave + 1) / NW;
  int s = s0;
  for (; s + U <= s1; s += U) {
    u32x4 xf[U], bfr[NT][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      xf[u] = *reinterpret_cast<const u32x4*>(xr + ((s + u) << 5));
#pragma unroll
      for (int t = 0; t < NT; ++t) bfr[t][u] = *reinterpret_cast<const u32x4*>(br[t] + ((s + u) << 5));
    }
    __builtin_amdgcn_sched_barrier(0);  // every load of the group is issued before the first product waits for one
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t] = mma16(xf[u], bfr[t][u], acc[t]);  // rows of X = MFMA rows, rows of Bm = columns
  }
  for (; s < s1; ++s) {
    const u32x4 xf = *reinterpret_cast<const u32x4*>(xr + (s << 5));
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = mma16(xf, *reinterpret_cast<const u32x4*>(br[t] + (s << 5)), acc[t]);
  }
  if (wave == NW - 1 && (K & 31)) {  // partial last step: lanes whose 8 k lie past K contribute zeros
    const int k = full << 5;
    const bool ok = k + g * 8 < K;
    const int kc = ok ? k : 0;
    u32x4 xf = *reinterpret_cast<const u32x4*>(xr + kc);
    if (!ok) xf = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = mma16(xf, *reinterpret_cast<const u32x4*>(br[t] + kc), acc[t]);
  }
  __shared__ float4 red[NW][NT][64];
#pragma unroll
  for (int t = 0; t < NT; ++t) red[wave][t][lane] = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
  __syncthreads();
  if (wave == 0) {
    bool over = false;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float4 sm = red[0][t][lane];
#pragma unroll
      for (int w = 1; w < NW; ++w) {
        const float4 o = red[w][t][lane];
        sm.x += o.x; sm.y += o.y; sm.z += o.z; sm.w += o.w;
      }
      // lane holds D[m = 4g + e][n = i16]
      const int n = t * 16 + i16;
      const float v[4] = {sm.x, sm.y, sm.z, sm.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + 4 * g + e;
        if (m < M && n < N) C[(long long)m * ldc + n] = F2EG(v[e] * alpha, over);
      }
    }
    elem_flag(over, flag);
  }
}

// ---------------------------------------------------------------- adapter gradients: G[j, r] += sum_t X[t, j] U[t, r]
// Two passes without atomics.  Pass 1: a workgroup covers 512 j x one token chunk; each thread owns two adjacent j
// and all R ranks.  The U rows are widened to fp32 in LDS 64 tokens at a time and read as wave-wide broadcasts; X is
// read as one 32-bit word per lane and token, eight tokens in flight (rows past the chunk reuse its last row against
// zero U rows).  The chunk's sums go to part[chunk][r][j].  Pass 2 adds the chunks and accumulates into G.
constexpr int kLgT = 64, kLgMaxChunks = 32;
// Half operands: two tokens per v_dot2_f32_f16 (exact products, fp32 accumulation).  U is staged in LDS as packed
// pairs (U[t][r], U[t+1][r]); the matching pairs of X are assembled from the two tokens' 32-bit words.
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
template <int R>
__global__ void __launch_bounds__(256) k_lora_grad_part(const bf* X, long long ldx, const bf* U, long long ldu, float* part,
                                                        int T, int J, int tpc) {
  __shared__ __align__(16) unsigned us2[kLgT / 2][R];
  const int tid = threadIdx.x;
  const int j0 = (blockIdx.x * 256 + tid) * 2;
  const int c0 = blockIdx.y * tpc, c1 = min(T, c0 + tpc);
  float a0[R], a1[R];
#pragma unroll
  for (int r = 0; r < R; ++r) a0[r] = a1[r] = 0.f;
  for (int t0 = c0; t0 < c1; t0 += kLgT) {
    const int nt = min(kLgT, c1 - t0);
    __syncthreads();
    for (int i = tid; i < (kLgT / 2) * R; i += 256) {
      const int tp = i / R, r = i - tp * R;
      const unsigned lo = 2 * tp < nt ? U[(long long)(t0 + 2 * tp) * ldu + r] : 0u;
      const unsigned hi = 2 * tp + 1 < nt ? U[(long long)(t0 + 2 * tp + 1) * ldu + r] : 0u;
      us2[tp][r] = lo | (hi << 16);
    }
    __syncthreads();
    const bf* xp = X + (long long)t0 * ldx + min(j0, J - 2);
    for (int tp = 0; tp < kLgT / 2; tp += 4) {
      unsigned xv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) xv[u] = *reinterpret_cast<const unsigned*>(xp + (long long)min(2 * tp + u, nt - 1) * ldx);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned w0 = xv[2 * u], w1 = xv[2 * u + 1];
        const h16x2 p0 = __builtin_bit_cast(h16x2, (w0 & 0xffffu) | (w1 << 16));        // (X[t][j0],   X[t+1][j0])
        const h16x2 p1 = __builtin_bit_cast(h16x2, (w0 >> 16) | (w1 & 0xffff0000u));   // (X[t][j0+1], X[t+1][j0+1])
#pragma unroll
        for (int r = 0; r < R; r += 4) {
          const uint4 uu = *reinterpret_cast<const uint4*>(&us2[tp + u][r]);
          const unsigned uw[4] = {uu.x, uu.y, uu.z, uu.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const h16x2 up = __builtin_bit_cast(h16x2, uw[e]);
            a0[r + e] = __builtin_amdgcn_fdot2(p0, up, a0[r + e], false);
            a1[r + e] = __builtin_amdgcn_fdot2(p1, up, a1[r + e], false);
          }
        }
      }
    }
  }
  if (j0 < J) {
    float* p = part + (long long)blockIdx.y * R * J + j0;
#pragma unroll
    for (int r = 0; r < R; ++r) *reinterpret_cast<float2*>(p + (long long)r * J) = make_float2(a0[r], a1[r]);
  }
}


// MFMA version of pass 1 for 16-byte aligned operands (J, ldx, ldu multiples of 8).  The product contracts over the
// ROW index of both operands (part[r][j] = sum_t X[t][j] U[t][r]), the layout MFMA operands do not come in: a lane must
// hold eight consecutive t of one column.  gfx950's transposing LDS read does that turn on the way out of LDS: with
// the tiles stored as they are in memory ([t][j], [t][r]) and lane q of every 16-lane group pointing at row q / 4,
// columns 4 (q % 4) .. + 3 of a 4 x 16 block, ds_read_b64_tr_b16 leaves lane i of the group with column i of the four
// rows -- two such reads give a lane its eight t of v_mfma_f32_16x16x32.  Workgroup: 256 columns j (64 per wave, four
// 16-column tiles) x all R ranks x one token chunk, 32 tokens per step through LDS.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned lg_u32x4 __attribute__((ext_vector_type(4)));  // native vector: arrays of HIP's uint4 struct were left in scratch memory
constexpr int kLmJ = 256, kLmT = 32, kLmPF = 4, kLmXS = kLmJ + 8;  // tile sizes, steps in flight; padded row of the X tile (halves)

template <int R>
__global__ void __launch_bounds__(256) k_lora_grad_mfma(LoraGradJobs jobs, float* part_all, int T) {
  const LoraGradJob& jb = jobs.j[blockIdx.z];
  if ((int)blockIdx.x >= jb.jt || (int)blockIdx.y >= jb.nch) return;  // the grid is sized for the largest job
  const bf* X = jb.X;
  const bf* U = jb.U;
  const long long ldx = jb.ldx, ldu = jb.ldu;
  const int J = jb.J, tpc = jb.tpm;
  float* part = part_all + jb.part_off;
  constexpr int RP = R < 16 ? 16 : R;  // rank padded to an MFMA tile (the padding columns of the U tile stay zero)
  constexpr int NT = RP / 16;          // 16-rank tiles
  constexpr int US = RP + 8;           // padded row of the U tile (halves)
  __shared__ __align__(16) unsigned short xs[kLmT][kLmXS];
  __shared__ __align__(16) unsigned short us[kLmT][US];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = blockIdx.x * kLmJ;
  const int c0 = blockIdx.y * tpc, c1 = min(T, c0 + tpc);
  f32x4 acc[4][NT];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int i = tid; i < kLmT * US; i += 256) (&us[0][0])[i] = 0;  // zero once: rows and columns never written stay zero

  // staging coordinates: X tile = 32 rows x 32 chunks of 16 bytes, four per thread; U tile = 32 rows x R / 8 chunks
  const int xc = tid & 31, xr = tid >> 5;
  const int xcol = min(j0 + xc * 8, J - 8);  // columns past J are loaded from a valid place and never stored
  constexpr int UCH = R / 8;
  const int uc = tid % UCH, ur = tid / UCH;  // threads with ur >= 32 stage nothing
  // fragment coordinates: 16-lane group g covers t = 8g .. 8g+7; lane q of it points at row q / 4, columns 4 (q % 4)
  const int g = lane >> 4, q = lane & 15;
  const int frow = 8 * g + (q >> 2), fcol = 4 * (q & 3);

  // kLmPF steps of loads are issued together (the MFMAs of a step take a fraction of a load's latency, so one step
  // of prefetch would leave every step waiting for memory)
  for (int tb = c0; tb < c1; tb += kLmT * kLmPF) {
    lg_u32x4 xv[kLmPF][4], uv[kLmPF];
#pragma unroll
    for (int p = 0; p < kLmPF; ++p) {
      const int t0 = tb + p * kLmT;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        xv[p][i] = *reinterpret_cast<const lg_u32x4*>(X + (long long)min(t0 + xr + 8 * i, T - 1) * ldx + xcol);
      // rows past the chunk are fetched from a valid row and zeroed below: they add nothing
      uv[p] = *reinterpret_cast<const lg_u32x4*>(U + (long long)min(t0 + min(ur, kLmT - 1), T - 1) * ldu + uc * 8);
    }
#pragma unroll
    for (int p = 0; p < kLmPF; ++p) {
      const int t0 = tb + p * kLmT;
      if (t0 >= c1) break;  // uniform
      __syncthreads();      // the previous step's fragments have been read
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<lg_u32x4*>(&xs[xr + 8 * i][xc * 8]) = xv[p][i];
      if (ur < kLmT) *reinterpret_cast<lg_u32x4*>(&us[ur][uc * 8]) = t0 + ur < c1 ? uv[p] : lg_u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
      s16x8 bfr[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(&us[frow][nt * 16 + fcol]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(&us[frow + 4][nt * 16 + fcol]));
        bfr[nt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        const int col = wave * 64 + mt * 16 + fcol;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(&xs[frow][col]));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(&xs[frow + 4][col]));
        const s16x8 afr = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, afr), __builtin_bit_cast(f16x8, bfr[nt]), acc[mt][nt], 0, 0, 0);
        }
      }
    }
  }
  // lane holds out[j = tile + 4 (lane / 16) + v][r = tile + lane % 16], v = 0..3: four consecutive j of one rank
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
    const int j = j0 + wave * 64 + mt * 16 + 4 * g;
    if (j >= J) continue;  // J % 8 == 0: the four columns are in or out together
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int r = nt * 16 + q;
      if (r < R)
        *reinterpret_cast<float4*>(part + (long long)blockIdx.y * R * J + (long long)r * J + j) =
            make_float4(acc[mt][nt][0], acc[mt][nt][1], acc[mt][nt][2], acc[mt][nt][3]);
    }
  }
}

// G[j*sj + r*sr] += out_mul * sum_c part[c][r][j]: one thread per (r, j), lanes along j (the reads of part, 2 x
// nchunk times the volume of G, are the contiguous side)
__global__ void __launch_bounds__(256) k_lora_grad_reduce(const float* part, int nchunk, float* G, long long sj, long long sr,
                                                          int J, long long RJ, const float* out_mul) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= RJ) return;
  const int r = (int)(i / J), j = (int)(i - (long long)r * J);
  float sum = 0.f;
#pragma unroll 8
  for (int c = 0; c < nchunk; ++c) sum += part[c * RJ + i];
  float* g = G + (long long)j * sj + (long long)r * sr;
  *g += sum * (out_mul ? *out_mul : 1.f);
}

__global__ void __launch_bounds__(256) k_lora_grad_reduce_multi(LoraGradJobs jobs, const float* part_all, int R, const float* out_mul) {
  const LoraGradJob& jb = jobs.j[blockIdx.y];
  const long long RJ = (long long)R * jb.J;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= RJ) return;
  const int r = (int)(i / jb.J), j = (int)(i - (long long)r * jb.J);
  const float* part = part_all + jb.part_off;
  float sum = 0.f;
  for (int c = 0; c < jb.nch; ++c) sum += part[c * RJ + i];
  float* g = jb.G + (long long)j * jb.sj + (long long)r * jb.sr;
  *g += sum * (out_mul ? *out_mul : 1.f);
}

__global__ void __launch_bounds__(256) k_sum_groups(const bf* in, bf* out, long long total, int n_kv, int G, int d, int* flag) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int kvd = n_kv * d;
  const long long t = i / kvd;
  const int rem = (int)(i - t * kvd), c = rem / d, e = rem - c * d;
  float s = 0.f;
  for (int g = 0; g < G; ++g) s += E2F(in[t * (long long)kvd * G + (c * G + g) * d + e]);
  bool over = false;
  out[i] = F2EG(s, over);
  elem_flag(over, flag);
}

__global__ void __launch_bounds__(256) k_convert_jobs(FtConvJobs jobs) {
  const FtConvJob jb = jobs.j[blockIdx.y];
  const long long n = (long long)jb.R * jb.C;
  bool over = false;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
    const unsigned short v = F2EG(jb.src_f32 ? static_cast<const float*>(jb.src)[i] : bf2f(static_cast<const bf*>(jb.src)[i]), over);
    if (jb.transpose) {
      const int r = (int)(i / jb.C), c = (int)(i - (long long)r * jb.C);
      jb.dst[(long long)c * jb.R + r] = v;
    } else {
      jb.dst[i] = v;
    }
  }
  elem_flag(over, jobs.flag);
}

inline unsigned nblk(long long n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

void ft_rmsnorm_fwd(const float* x, const float* g, bf* h, float* rho, int T, int H, float eps, int* flag, hipStream_t st) {
  hipLaunchKernelGGL(k_rmsnorm_fwd, dim3(T), dim3(256), 0, st, x, g, h, rho, H, eps, flag);
}
void ft_rmsnorm_bwd(const float* dh, const float* x, const float* rho, const float* g, const float* dres, float* dx, bf* dx16,
                    int T, int H, const float* res_mul, const float* out_mul, int* flag, hipStream_t st) {
  hipLaunchKernelGGL(k_rmsnorm_bwd, dim3(T), dim3(256), 0, st, dh, x, rho, g, dres, dx, dx16, H, res_mul, out_mul, flag);
}
void ft_rope(bf* t, int T, int S, int heads, int d, const double* inv_freq, bool inverse, int* flag, hipStream_t st) {
  hipLaunchKernelGGL(k_rope, dim3(T), dim3(256), 0, st, t, S, heads, d, inv_freq, inverse ? -1.f : 1.f, flag);
}
void ft_convert_jobs(const FtConvJobs& jobs, hipStream_t st) {
  hipLaunchKernelGGL(k_convert_jobs, dim3(64, jobs.n), dim3(256), 0, st, jobs);
}
void ft_scale_to_e(const float* x, bf* y, long long n, float* scale, int parity, int target_log2, hipStream_t st) {
  unsigned* bits = reinterpret_cast<unsigned*>(scale + 2);
  hipLaunchKernelGGL(k_amax, dim3(std::min(nblk(n / 4, 1024), 1024u)), dim3(256), 0, st, x, n / 4, bits + (parity & 1));
  hipLaunchKernelGGL(k_f32_to_e_scaled, dim3(nblk(n / 4, 256)), dim3(256), 0, st, x, y, n / 4, bits + (parity & 1),
                     bits + ((parity & 1) ^ 1), scale, target_log2);
}
void ft_transpose_heads(const TransposeJobs& jobs, int Bf, int S, hipStream_t st) {
  if (jobs.n < 1) return;
  int cmax = 0;
  for (int i = 0; i < jobs.n; ++i) cmax = std::max(cmax, jobs.C[i]);
  hipLaunchKernelGGL(k_transpose_heads, dim3((cmax + 63) / 64, (S + 63) / 64, Bf * jobs.n), dim3(256), 0, st, jobs, Bf, S);
}
void ft_skinny_nt_multi(const SkinnyNtJobs& jobs, int M, float alpha, int* flag, hipStream_t st) {
  if (jobs.n < 1) return;
  int nmax = 0;
  for (int i = 0; i < jobs.n; ++i) nmax = std::max(nmax, jobs.j[i].N);
  const int nt = (nmax + 15) / 16;  // jobs with fewer columns mask their stores
  const dim3 grid((M + 15) / 16, jobs.n), blk(512);
  if (nt == 1) hipLaunchKernelGGL(k_skinny_nt<1>, grid, blk, 0, st, jobs, M, alpha, flag);
  else if (nt == 2) hipLaunchKernelGGL(k_skinny_nt<2>, grid, blk, 0, st, jobs, M, alpha, flag);
  else hipLaunchKernelGGL(k_skinny_nt<4>, grid, blk, 0, st, jobs, M, alpha, flag);
}
// floats of partial sums one job of the MFMA path can need: nch * J with nch <= max(1, 512 / column tiles)
static size_t lora_grad_job_floats(int J, int R) { return (size_t)std::max(512 * kLmJ, (J + kLmJ - 1) / kLmJ * kLmJ) * R; }
size_t ft_lora_grad_ws_floats(int J, int R) {
  return std::max((size_t)kLgMaxChunks * J * R, (size_t)kLoraGradMaxJobs * lora_grad_job_floats(J, R));
}
template <int R>
static void lora_grad_launch(const bf* X, long long ldx, const bf* U, long long ldu, float* G, long long sj, long long sr, int T,
                             int J, const float* out_mul, float* part, hipStream_t st) {
  const int tpc = std::max(kLgT, ((T + kLgMaxChunks - 1) / kLgMaxChunks + kLgT - 1) / kLgT * kLgT);
  const int nchunk = (T + tpc - 1) / tpc;
  hipLaunchKernelGGL(k_lora_grad_part<R>, dim3((J + 511) / 512, nchunk), dim3(256), 0, st, X, ldx, U, ldu, part, T, J, tpc);
  hipLaunchKernelGGL(k_lora_grad_reduce, dim3(nblk((long long)R * J, 256)), dim3(256), 0, st, part, nchunk, G, sj, sr, J, (long long)R * J,
                     out_mul);
}
static void lora_grad_vector(const LoraGradJob& b, int T, int R, const float* out_mul, float* part, hipStream_t st) {
  if (R == 8) lora_grad_launch<8>(b.X, b.ldx, b.U, b.ldu, b.G, b.sj, b.sr, T, b.J, out_mul, part, st);
  else if (R == 16) lora_grad_launch<16>(b.X, b.ldx, b.U, b.ldu, b.G, b.sj, b.sr, T, b.J, out_mul, part, st);
  else if (R == 32) lora_grad_launch<32>(b.X, b.ldx, b.U, b.ldu, b.G, b.sj, b.sr, T, b.J, out_mul, part, st);
  else lora_grad_launch<64>(b.X, b.ldx, b.U, b.ldu, b.G, b.sj, b.sr, T, b.J, out_mul, part, st);
}
void ft_lora_grad_multi(LoraGradJobs& jobs, int T, int R, const float* out_mul, float* part, hipStream_t st) {
  if (jobs.n < 1) return;
  bool aligned = (reinterpret_cast<uintptr_t>(part) & 15) == 0;
  for (int i = 0; i < jobs.n; ++i) {
    const LoraGradJob& b = jobs.j[i];
    aligned = aligned && b.J % 8 == 0 && b.ldx % 8 == 0 && b.ldu % 8 == 0 &&
              ((reinterpret_cast<uintptr_t>(b.X) | reinterpret_cast<uintptr_t>(b.U)) & 15) == 0;
  }
  if (!aligned) {  // the vector kernels, one job after the other (each uses the whole scratch)
    for (int i = 0; i < jobs.n; ++i) lora_grad_vector(jobs.j[i], T, R, out_mul, part, st);
    return;
  }
  // about two workgroups per compute unit per job and whole groups of steps in flight
  int max_jt = 0, max_nch = 0, max_j = 0;
  long long off = 0;
  const int unit = kLmT * kLmPF;
  for (int i = 0; i < jobs.n; ++i) {
    LoraGradJob& b = jobs.j[i];
    b.jt = (b.J + kLmJ - 1) / kLmJ;
    const int want = std::min(kLgMaxChunks, std::max(1, 512 / b.jt));
    b.tpm = std::max(unit, ((T + want - 1) / want + unit - 1) / unit * unit);
    b.nch = (T + b.tpm - 1) / b.tpm;
    b.part_off = off;
    off += (long long)lora_grad_job_floats(b.J, R);
    max_jt = std::max(max_jt, b.jt);
    max_nch = std::max(max_nch, b.nch);
    max_j = std::max(max_j, b.J);
  }
  const dim3 grid(max_jt, max_nch, jobs.n);
  if (R == 8) hipLaunchKernelGGL(k_lora_grad_mfma<8>, grid, dim3(256), 0, st, jobs, part, T);
  else if (R == 16) hipLaunchKernelGGL(k_lora_grad_mfma<16>, grid, dim3(256), 0, st, jobs, part, T);
  else if (R == 32) hipLaunchKernelGGL(k_lora_grad_mfma<32>, grid, dim3(256), 0, st, jobs, part, T);
  else hipLaunchKernelGGL(k_lora_grad_mfma<64>, grid, dim3(256), 0, st, jobs, part, T);
  hipLaunchKernelGGL(k_lora_grad_reduce_multi, dim3(nblk((long long)R * max_j, 256), jobs.n), dim3(256), 0, st, jobs, part, R, out_mul);
}
void ft_lora_grad(const bf* X, long long ldx, const bf* U, long long ldu, float* G, long long sj, long long sr, int T, int J,
                  int R, const float* out_mul, float* part, hipStream_t st) {
  LoraGradJobs jobs{};
  jobs.n = 1;
  jobs.j[0] = LoraGradJob{X, ldx, U, ldu, G, sj, sr, J, 0, 0, 0, 0};
  ft_lora_grad_multi(jobs, T, R, out_mul, part, st);
}
void ft_sum_groups(const bf* in, bf* out, int T, int n_kv, int G, int d, int* flag, hipStream_t st) {
  const long long total = (long long)T * n_kv * d;
  hipLaunchKernelGGL(k_sum_groups, dim3(nblk(total, 256)), dim3(256), 0, st, in, out, total, n_kv, G, d, flag);
}

}  // namespace harli
