// Fused causal attention for the finetune unit on gfx950 (the attention part of the layer forward / backward
// that the per-layer finetune unit of Harli Sec. 6.1 runs; scores never leave the chip).
//
// All three kernels use v_mfma_f32_32x32x16 with one operand held in registers for the whole kernel and the
// other streamed through LDS in blocks of 64 rows.  The accumulator layout of a 32x32 tile (lane = column,
// registers = rows 8*(v/4) + 4*(lane/32) + v%4) decides the orientation of every product:
//   * forward and dQ compute S^T = K Q^T, so that a lane owns ONE query: its running max / sum (forward) or its
//     lse / delta (backward) are per-lane scalars, and the probabilities leave the accumulator already in the
//     layout of a B operand whose contraction index is the key;
//   * dK / dV compute S = Q K^T, so that a lane owns one key and the probabilities are a B operand whose
//     contraction index is the query.
// In both cases the second product contracts over the index held in the accumulator's REGISTERS.  Register v of a
// lane half h is contraction slot v%8 of MFMA step v/8, i.e. row 16*(v/8) + 8*((v%8)/4) + 4h + v%4: the A operand
// of the second product (a transposed tile V^T, K^T, Q^T or dO^T in LDS) is read with the same permutation, as
// two 8-byte pieces at columns 4h and 8 + 4h of each 16-column step.  No data moves between lanes.
#include "ft_attention.h"

#include "ft_elem.h"

namespace harli {
namespace {

constexpr int KB = 64;            // rows of the streamed operand per block
constexpr int TS = KB * 2 + 16;   // byte stride of a transposed tile row (64 columns + pad)
// native vector types: arrays of them stay in registers (arrays of the HIP uint4 struct were left in scratch)
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;
typedef unsigned __attribute__((ext_vector_type(2))) u32x2;
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mma32(const u32x4& a, const u32x4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// A fragment of a row-major LDS tile (row stride RS bytes): rows sub*32 + lane%32, k = 16j + 8h .. +7
template <int RS>
__device__ __forceinline__ u32x4 frag_rows(const char* tile, int sub, int j, int l31, int h) {
  return *reinterpret_cast<const u32x4*>(tile + (sub * 32 + l31) * RS + (16 * j + 8 * h) * 2);
}
// A fragment of a transposed LDS tile [rows e][64 columns]: row et*32 + lane%32, columns of step (sub, jj) in the
// accumulator-register order (see the file header)
__device__ __forceinline__ u32x4 frag_cols(const char* tile, int et, int sub, int jj, int l31, int h) {
  const char* p = tile + (et * 32 + l31) * TS + (sub * 32 + 16 * jj + 4 * h) * 2;
  const u32x2 lo = *reinterpret_cast<const u32x2*>(p), hi = *reinterpret_cast<const u32x2*>(p + 16);
  return u32x4{lo.x, lo.y, hi.x, hi.y};
}
__device__ __forceinline__ u32x4 pack8(const f32x16& a, int o) {
  return u32x4{PACK2(a[o], a[o + 1]), PACK2(a[o + 2], a[o + 3]), PACK2(a[o + 4], a[o + 5]), PACK2(a[o + 6], a[o + 7])};
}
__device__ __forceinline__ f32x16 zero16f() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; ++v) z[v] = 0.f;
  return z;
}

// -------------------------------------------------------------------------------------------- forward
// grid (ceil(S/128), Bf*n_q); a workgroup owns 128 queries of one head, wave w the 32 queries 32w..32w+31.
template <int D>
__global__ void __launch_bounds__(256, 2) k_attn_fwd(const bf* __restrict__ q, const bf* __restrict__ k, const bf* __restrict__ vT,
                                                  bf* __restrict__ o, float* __restrict__ lse, int S, int nq, int nkv,
                                                  float scale_log2) {
  constexpr int RS = D * 2 + 16, NJ = D / 16, NE = D / 32, CPT = D / 32;
  extern __shared__ __align__(16) char smem[];
  char* sK = smem;             // [KB][D] keys x head_dim
  char* sV = smem + KB * RS;   // [D][KB] head_dim x keys
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, h = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;  // the blocks with the longest causal span first
  const int z = blockIdx.y, b = z / nq, head = z - b * nq, hk = head / (nq / nkv);
  const int QD = nq * D, KVD = nkv * D;
  const int q0 = qb * 128 + wave * 32, qrow = q0 + l31, qc = min(qrow, S - 1);

  u32x4 Qf[NJ];
  {
    const bf* qp = q + ((long long)b * S + qc) * QD + head * D + 8 * h;
#pragma unroll
    for (int j = 0; j < NJ; ++j) Qf[j] = *reinterpret_cast<const u32x4*>(qp + 16 * j);
  }
  f32x16 O[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) O[e] = zero16f();
  float m_run = -INFINITY, l_run = 0.f;

  const int nkb = min(qb * 128 + 127, S - 1) / KB + 1;
  const bf* kbase = k + (long long)b * S * KVD + hk * D;
  const bf* vbase = vT + (long long)(b * nkv + hk) * D * S;
  // per-thread chunk coordinates of the two tiles (CPT 16-byte chunks each)
  u32x4 pk[CPT], pv[CPT];
#define FWD_FETCH(kb_)                                                                                        \
  _Pragma("unroll") for (int i = 0; i < CPT; ++i) {                                                           \
    const int c = tid + 256 * i;                                                                              \
    const int kr = c / (D / 8), kc = c - kr * (D / 8);                                                        \
    pk[i] = *reinterpret_cast<const u32x4*>(kbase + (long long)min((kb_) * KB + kr, S - 1) * KVD + kc * 8);   \
    const int ve = c >> 3, vc = c & 7;                                                                        \
    pv[i] = *reinterpret_cast<const u32x4*>(vbase + (long long)ve * S + min((kb_) * KB + vc * 8, S - 8));     \
  }
  FWD_FETCH(0)
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + 256 * i;
      const int kr = c / (D / 8), kc = c - kr * (D / 8);
      *reinterpret_cast<u32x4*>(sK + kr * RS + kc * 16) = pk[i];
      const int ve = c >> 3, vc = c & 7;
      *reinterpret_cast<u32x4*>(sV + ve * TS + vc * 16) = pv[i];
    }
    __syncthreads();
    if (kb + 1 < nkb) { FWD_FETCH(kb + 1) }
    if (kb * KB > q0 + 31) continue;  // every key of the block is past this wave's queries
    f32x16 sc[2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      sc[sub] = zero16f();
#pragma unroll
      for (int j = 0; j < NJ; ++j) sc[sub] = mma32(frag_rows<RS>(sK, sub, j, l31, h), Qf[j], sc[sub]);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = kb * KB + sub * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        const float s = key > qrow ? -INFINITY : sc[sub][v] * scale_log2;
        sc[sub][v] = s;
        mx = fmaxf(mx, s);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // finite: block 0 holds key 0 <= every query, and later blocks inherit a finite running maximum
    const float m_new = fmaxf(m_run, mx);
    const float alpha = exp2f(m_run - m_new);
    float rs = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = exp2f(sc[sub][v] - m_new);
        sc[sub][v] = p;
        rs += p;
      }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * alpha + rs;
    m_run = m_new;
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int v = 0; v < 16; ++v) O[e][v] *= alpha;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const u32x4 pf = pack8(sc[sub], 8 * jj);
#pragma unroll
        for (int e = 0; e < NE; ++e) O[e] = mma32(frag_cols(sV, e, sub, jj, l31, h), pf, O[e]);
      }
  }
#undef FWD_FETCH
  if (qrow < S) {
    const float inv = 1.f / l_run;
    bf* op = o + ((long long)b * S + qrow) * QD + head * D;
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(op + e * 32 + 8 * g + 4 * h) =
            u32x2{PACK2(O[e][4 * g] * inv, O[e][4 * g + 1] * inv), PACK2(O[e][4 * g + 2] * inv, O[e][4 * g + 3] * inv)};
    if (h == 0) lse[(long long)z * S + qrow] = (m_run + log2f(l_run)) * kLn2;
  }
}

// -------------------------------------------------------------------------------------------- backward: dQ
// grid (ceil(S/128), Bf*n_q); same ownership as the forward kernel.  dQ^T[e][q] += K^T[e][k] dS^T[k][q].
// Also computes delta[q] = sum_e dO[q][e] O[q][e] and stores it.
template <int D>
__global__ void __launch_bounds__(256, 2) k_attn_bwd_dq(const bf* __restrict__ q, const bf* __restrict__ k, const bf* __restrict__ v,
                                                     const bf* __restrict__ kT, const bf* __restrict__ dO,
                                                     const bf* __restrict__ o, const float* __restrict__ lse,
                                                     float* __restrict__ delta, bf* __restrict__ dq, int S, int nq, int nkv,
                                                     float scale, float scale_log2, int* flag) {
  constexpr int RS = D * 2 + 16, NJ = D / 16, NE = D / 32, CPT = D / 32;
  extern __shared__ __align__(16) char smem[];
  char* sK = smem;                  // [KB][D]
  char* sV = smem + KB * RS;        // [KB][D]
  char* sKT = smem + 2 * KB * RS;   // [D][KB]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, h = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int z = blockIdx.y, b = z / nq, head = z - b * nq, hk = head / (nq / nkv);
  const int QD = nq * D, KVD = nkv * D;
  const int q0 = qb * 128 + wave * 32, qrow = q0 + l31, qc = min(qrow, S - 1);

  u32x4 Qf[NJ], Gf[NJ];  // this lane's query row and its dO row as B operands
  {
    const long long ro = ((long long)b * S + qc) * QD + head * D + 8 * h;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      Qf[j] = *reinterpret_cast<const u32x4*>(q + ro + 16 * j);
      Gf[j] = *reinterpret_cast<const u32x4*>(dO + ro + 16 * j);
    }
  }
  const float lse2 = lse[(long long)z * S + qc] * kLog2e;
  // delta = rowsum(dO * O) of this lane's query: the lane holds half of the row's dO (8 of every 16 elements), its
  // partner lane the other half.  Stored for the dK / dV kernel, which runs after this one.
  float dl = 0.f;
  {
    const bf* op = o + ((long long)b * S + qc) * QD + head * D + 8 * h;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const u32x4 ov = *reinterpret_cast<const u32x4*>(op + 16 * j);
      float gf[8], of[8];
      UNPACK8(uint4{Gf[j].x, Gf[j].y, Gf[j].z, Gf[j].w}, gf);
      UNPACK8(uint4{ov.x, ov.y, ov.z, ov.w}, of);
#pragma unroll
      for (int e = 0; e < 8; ++e) dl += gf[e] * of[e];
    }
    dl += __shfl_xor(dl, 32, 64);
    if (h == 0 && qrow < S) delta[(long long)z * S + qrow] = dl;
  }
  f32x16 dQ[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) dQ[e] = zero16f();

  const int nkb = min(qb * 128 + 127, S - 1) / KB + 1;
  const bf* kbase = k + (long long)b * S * KVD + hk * D;
  const bf* vbase = v + (long long)b * S * KVD + hk * D;
  const bf* ktbase = kT + (long long)(b * nkv + hk) * D * S;
  u32x4 pk[CPT], pv[CPT], pt[CPT];
#define DQ_FETCH(kb_)                                                                                         \
  _Pragma("unroll") for (int i = 0; i < CPT; ++i) {                                                           \
    const int c = tid + 256 * i;                                                                              \
    const int kr = c / (D / 8), kc = c - kr * (D / 8);                                                        \
    const long long ro = (long long)min((kb_) * KB + kr, S - 1) * KVD + kc * 8;                               \
    pk[i] = *reinterpret_cast<const u32x4*>(kbase + ro);                                                      \
    pv[i] = *reinterpret_cast<const u32x4*>(vbase + ro);                                                      \
    const int te = c >> 3, tc = c & 7;                                                                        \
    pt[i] = *reinterpret_cast<const u32x4*>(ktbase + (long long)te * S + min((kb_) * KB + tc * 8, S - 8));    \
  }
  DQ_FETCH(0)
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + 256 * i;
      const int kr = c / (D / 8), kc = c - kr * (D / 8);
      *reinterpret_cast<u32x4*>(sK + kr * RS + kc * 16) = pk[i];
      *reinterpret_cast<u32x4*>(sV + kr * RS + kc * 16) = pv[i];
      const int te = c >> 3, tc = c & 7;
      *reinterpret_cast<u32x4*>(sKT + te * TS + tc * 16) = pt[i];
    }
    __syncthreads();
    if (kb + 1 < nkb) { DQ_FETCH(kb + 1) }
    if (kb * KB > q0 + 31) continue;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x16 sc = zero16f(), dp = zero16f();
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        sc = mma32(frag_rows<RS>(sK, sub, j, l31, h), Qf[j], sc);
        dp = mma32(frag_rows<RS>(sV, sub, j, l31, h), Gf[j], dp);
      }
#pragma unroll
      for (int vv = 0; vv < 16; ++vv) {
        const int key = kb * KB + sub * 32 + 8 * (vv >> 2) + 4 * h + (vv & 3);
        const float p = key > qrow ? 0.f : exp2f(sc[vv] * scale_log2 - lse2);
        sc[vv] = p * (dp[vv] - dl);
      }
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const u32x4 df = pack8(sc, 8 * jj);
#pragma unroll
        for (int e = 0; e < NE; ++e) dQ[e] = mma32(frag_cols(sKT, e, sub, jj, l31, h), df, dQ[e]);
      }
    }
  }
#undef DQ_FETCH
  if (qrow < S) {
    bf* op = dq + ((long long)b * S + qrow) * QD + head * D;
    bool over = false;
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<u32x2*>(op + e * 32 + 8 * g + 4 * h) = u32x2{PACK2G(dQ[e][4 * g] * scale, dQ[e][4 * g + 1] * scale, over),
                                                                       PACK2G(dQ[e][4 * g + 2] * scale, dQ[e][4 * g + 3] * scale, over)};
    elem_flag(over, flag);
  }
}

// -------------------------------------------------------------------------------------------- backward: dK, dV
// grid (ceil(S/128), Bf*n_q); a workgroup owns 128 keys as seen by one QUERY head, wave w the keys 32w..32w+31, and
// streams the queries from its first key to the end of the sequence.
//   dV^T[e][k] += dO^T[e][q] P[q][k],   dK^T[e][k] += Q^T[e][q] dS[q][k]
template <int D>
__global__ void __launch_bounds__(256) k_attn_bwd_dkv(const bf* __restrict__ q, const bf* __restrict__ k, const bf* __restrict__ v,
                                                      const bf* __restrict__ qT, const bf* __restrict__ dO,
                                                      const bf* __restrict__ dOT, const float* __restrict__ lse,
                                                      const float* __restrict__ delta, bf* __restrict__ dkq,
                                                      bf* __restrict__ dvq, int S, int nq, int nkv, float scale,
                                                      float scale_log2, int* flag) {
  constexpr int RS = D * 2 + 16, NJ = D / 16, NE = D / 32, CPT = D / 32;
  extern __shared__ __align__(16) char smem[];
  char* sQ = smem;                              // [KB][D] queries x head_dim
  char* sG = smem + KB * RS;                    // [KB][D] dO
  char* sQT = smem + 2 * KB * RS;               // [D][KB]
  char* sGT = smem + 2 * KB * RS + D * TS;      // [D][KB]
  float* sL = reinterpret_cast<float*>(smem + 2 * KB * RS + 2 * D * TS);  // [KB] lse * log2(e), then [KB] delta
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, h = lane >> 5;
  const int kvb = blockIdx.x;  // block 0 has the longest span of queries and starts first
  const int z = blockIdx.y, b = z / nq, head = z - b * nq, hk = head / (nq / nkv);
  const int QD = nq * D, KVD = nkv * D;
  const int k0 = kvb * 128 + wave * 32, krow = k0 + l31, kc_ = min(krow, S - 1);

  u32x4 Kf[NJ], Vf[NJ];  // this lane's key and value rows as B operands
  {
    const long long ro = ((long long)b * S + kc_) * KVD + hk * D + 8 * h;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      Kf[j] = *reinterpret_cast<const u32x4*>(k + ro + 16 * j);
      Vf[j] = *reinterpret_cast<const u32x4*>(v + ro + 16 * j);
    }
  }
  f32x16 dV[NE], dK[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) dV[e] = zero16f(), dK[e] = zero16f();

  const int qb0 = kvb * 128 / KB, nqb = (S + KB - 1) / KB;
  const bf* qbase = q + (long long)b * S * QD + head * D;
  const bf* gbase = dO + (long long)b * S * QD + head * D;
  const bf* qtbase = qT + (long long)(b * nq + head) * D * S;
  const bf* gtbase = dOT + (long long)(b * nq + head) * D * S;
  const float* lbase = lse + (long long)z * S;
  const float* dbase = delta + (long long)z * S;
  u32x4 pq[CPT], pg[CPT], pqt[CPT], pgt[CPT];
  float pl;
#define KV_FETCH(qb_)                                                                                          \
  _Pragma("unroll") for (int i = 0; i < CPT; ++i) {                                                            \
    const int c = tid + 256 * i;                                                                               \
    const int rr = c / (D / 8), rc = c - rr * (D / 8);                                                         \
    const long long ro = (long long)min((qb_) * KB + rr, S - 1) * QD + rc * 8;                                 \
    pq[i] = *reinterpret_cast<const u32x4*>(qbase + ro);                                                       \
    pg[i] = *reinterpret_cast<const u32x4*>(gbase + ro);                                                       \
    const int te = c >> 3, tc = c & 7;                                                                         \
    const long long to = (long long)te * S + min((qb_) * KB + tc * 8, S - 8);                                  \
    pqt[i] = *reinterpret_cast<const u32x4*>(qtbase + to);                                                     \
    pgt[i] = *reinterpret_cast<const u32x4*>(gtbase + to);                                                     \
  }                                                                                                            \
  {                                                                                                            \
    const int r = min((qb_) * KB + (tid & 63), S - 1);                                                         \
    pl = tid < 64 ? lbase[r] * kLog2e : dbase[r];                                                              \
  }
  KV_FETCH(qb0)
  for (int qb = qb0; qb < nqb; ++qb) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + 256 * i;
      const int rr = c / (D / 8), rc = c - rr * (D / 8);
      *reinterpret_cast<u32x4*>(sQ + rr * RS + rc * 16) = pq[i];
      *reinterpret_cast<u32x4*>(sG + rr * RS + rc * 16) = pg[i];
      const int te = c >> 3, tc = c & 7;
      *reinterpret_cast<u32x4*>(sQT + te * TS + tc * 16) = pqt[i];
      *reinterpret_cast<u32x4*>(sGT + te * TS + tc * 16) = pgt[i];
    }
    if (tid < 128) sL[tid] = pl;
    __syncthreads();
    if (qb + 1 < nqb) { KV_FETCH(qb + 1) }
    if (qb * KB + KB - 1 < k0) continue;  // every query of the block precedes this wave's keys
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x16 sc = zero16f(), dp = zero16f();
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        sc = mma32(frag_rows<RS>(sQ, sub, j, l31, h), Kf[j], sc);
        dp = mma32(frag_rows<RS>(sG, sub, j, l31, h), Vf[j], dp);
      }
      // rows of the accumulator are queries: their lse and delta come in runs of four
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 l4 = *reinterpret_cast<const float4*>(sL + sub * 32 + 8 * g + 4 * h);
        const float4 d4 = *reinterpret_cast<const float4*>(sL + KB + sub * 32 + 8 * g + 4 * h);
        const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, ds[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int vv = 4 * g + c;
          const int qg = qb * KB + sub * 32 + 8 * g + 4 * h + c;
          const float p = (qg < krow || qg >= S) ? 0.f : exp2f(sc[vv] * scale_log2 - ls[c]);
          sc[vv] = p;
          dp[vv] = p * (dp[vv] - ds[c]);
        }
      }
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const u32x4 pf = pack8(sc, 8 * jj), df = pack8(dp, 8 * jj);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
          dV[e] = mma32(frag_cols(sGT, e, sub, jj, l31, h), pf, dV[e]);
          dK[e] = mma32(frag_cols(sQT, e, sub, jj, l31, h), df, dK[e]);
        }
      }
    }
  }
#undef KV_FETCH
  if (krow < S) {
    const long long ro = ((long long)b * S + krow) * QD + head * D;
    bool over = false;
#pragma unroll
    for (int e = 0; e < NE; ++e)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int eo = e * 32 + 8 * g + 4 * h;
        *reinterpret_cast<u32x2*>(dvq + ro + eo) =
            u32x2{PACK2G(dV[e][4 * g], dV[e][4 * g + 1], over), PACK2G(dV[e][4 * g + 2], dV[e][4 * g + 3], over)};
        *reinterpret_cast<u32x2*>(dkq + ro + eo) = u32x2{PACK2G(dK[e][4 * g] * scale, dK[e][4 * g + 1] * scale, over),
                                                         PACK2G(dK[e][4 * g + 2] * scale, dK[e][4 * g + 3] * scale, over)};
      }
    elem_flag(over, flag);
  }
}

template <int D>
constexpr int fwd_lds() { return KB * (D * 2 + 16) + D * TS; }
template <int D>
constexpr int dq_lds() { return 2 * KB * (D * 2 + 16) + D * TS; }
template <int D>
constexpr int dkv_lds() { return 2 * KB * (D * 2 + 16) + 2 * D * TS + 2 * KB * 4; }

template <int D>
harli_status set_attrs() {
  static bool done = false;
  if (done) return HARLI_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_fwd<D>), hipFuncAttributeMaxDynamicSharedMemorySize, fwd_lds<D>()) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bwd_dq<D>), hipFuncAttributeMaxDynamicSharedMemorySize, dq_lds<D>()) != hipSuccess ||
      hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_bwd_dkv<D>), hipFuncAttributeMaxDynamicSharedMemorySize, dkv_lds<D>()) != hipSuccess)
    return fail(HARLI_ERR_HIP, "attention: could not raise the dynamic LDS limit");
  done = true;
  return HARLI_OK;
}

harli_status check_shape(int Bf, int S, int nq, int nkv, int d) {
  if (!ft_attn_supported(d)) return fail(HARLI_ERR_INVALID, "attention: head_dim %d is not 64 or 128", d);
  if (Bf < 1 || S < 8 || (S & 7) || nq < 1 || nkv < 1 || nq % nkv) return fail(HARLI_ERR_INVALID, "attention: bad shape");
  return HARLI_OK;
}

}  // namespace

harli_status ft_attn_fwd(const bf* q, const bf* k, const bf* vT, bf* o, float* lse, int Bf, int S, int n_q, int n_kv, int d,
                         hipStream_t st) {
  harli_status s = check_shape(Bf, S, n_q, n_kv, d);
  if (s != HARLI_OK) return s;
  const dim3 grid((S + 127) / 128, Bf * n_q), blk(256);
  const float sl2 = kLog2e / sqrtf((float)d);
  if (d == 128) {
    if ((s = set_attrs<128>()) != HARLI_OK) return s;
    hipLaunchKernelGGL(k_attn_fwd<128>, grid, blk, fwd_lds<128>(), st, q, k, vT, o, lse, S, n_q, n_kv, sl2);
  } else {
    if ((s = set_attrs<64>()) != HARLI_OK) return s;
    hipLaunchKernelGGL(k_attn_fwd<64>, grid, blk, fwd_lds<64>(), st, q, k, vT, o, lse, S, n_q, n_kv, sl2);
  }
  return HARLI_OK;
}

harli_status ft_attn_bwd(const bf* q, const bf* k, const bf* v, const bf* o, const bf* qT, const bf* kT, const bf* dO,
                         const bf* dOT, const float* lse, float* delta, bf* dq, bf* dkq, bf* dvq, int Bf, int S, int n_q,
                         int n_kv, int d, int* flag, hipStream_t st) {
  harli_status s = check_shape(Bf, S, n_q, n_kv, d);
  if (s != HARLI_OK) return s;
  const dim3 grid((S + 127) / 128, Bf * n_q), blk(256);
  const float sc = 1.f / sqrtf((float)d), sl2 = kLog2e * sc;
  if (d == 128) {
    if ((s = set_attrs<128>()) != HARLI_OK) return s;
    hipLaunchKernelGGL(k_attn_bwd_dq<128>, grid, blk, dq_lds<128>(), st, q, k, v, kT, dO, o, lse, delta, dq, S, n_q, n_kv, sc, sl2, flag);
    hipLaunchKernelGGL(k_attn_bwd_dkv<128>, grid, blk, dkv_lds<128>(), st, q, k, v, qT, dO, dOT, lse, delta, dkq, dvq, S, n_q,
                       n_kv, sc, sl2, flag);
  } else {
    if ((s = set_attrs<64>()) != HARLI_OK) return s;
    hipLaunchKernelGGL(k_attn_bwd_dq<64>, grid, blk, dq_lds<64>(), st, q, k, v, kT, dO, o, lse, delta, dq, S, n_q, n_kv, sc, sl2, flag);
    hipLaunchKernelGGL(k_attn_bwd_dkv<64>, grid, blk, dkv_lds<64>(), st, q, k, v, qT, dO, dOT, lse, delta, dkq, dvq, S, n_q,
                       n_kv, sc, sl2, flag);
  }
  return HARLI_OK;
}

}  // namespace harli
