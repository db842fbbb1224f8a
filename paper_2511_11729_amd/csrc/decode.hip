// Decode step for gfx950 (Harli Sec. 2.1: one new token per sequence per step,
// reusing the KV cache; Sec. 2.2.1: the step is bound by DRAM bandwidth -- its
// GEMMs have M = batch -- so every kernel here is built around streaming the
// weights and the paged KV cache from HBM exactly once).
//
// Per layer, bf16 storage:
//   skinny<QKV>     h W{q,k,v}^T, x rho, rotary embedding, q -> workspace, k/v -> KV pages
//   paged_attn      split-KV attention over the page table + last-arriver merge
//   skinny<RESID>   x1 = x + o Wo^T, next operand bf16(x1*g2), sum x1^2
//   skinny<GATEUP>  m = silu(rho h2 Wg^T) * (rho h2 Wu^T)
//   skinny<RESID>   y = x1 + m Wd^T, operand and sum of squares for the next layer
// RMSNorm is folded: the GEMM operand is bf16(x*g) and the per-row factor
// rho = rsqrt(mean x^2 + eps) multiplies the fp32 accumulator afterwards.
//
// The skinny GEMM keeps the batch (<= 64 rows per pass) as the MFMA "column"
// operand and streams 16-row weight tiles as the "row" operand of
// v_mfma_f32_16x16x32_bf16; the K range is split over the waves of a
// workgroup and reduced through LDS, so epilogues see complete sums.
#include "ctx.h"
#include "device_utils.h"

using namespace harli;

namespace {

constexpr int kChunkTokens = 256;  // tokens per attention workgroup
constexpr int kPageTokens = 16;

enum { MODE_QKV = 0, MODE_RESID = 1, MODE_GATEUP = 2, MODE_LM = 3 };

struct SkinnyArgs {
  const unsigned short* x;  // [rows][K] bf16 operand; row jb is batch entry jb
  int B, b0, K;             // batch size, first batch row of this pass, contraction length
  int n_rows;               // output rows per weight matrix (tail masking)
  const unsigned short *w0, *w1, *w2;
  const float* ssq_in;      // sum of squares of the operand's source row (rho), or null
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
  // RESID
  const float* res;
  float* out;
  const float* gnext;
  unsigned short* hxn;
  float* ssq_out;
  // GATEUP
  unsigned short* mbuf;
  // LM
  float* logits;
};

template <int MODE>
struct ModeTraits {
  static constexpr int RT = (MODE == MODE_RESID) ? 1 : 2;
};

__device__ __forceinline__ uint4 ld16(const unsigned short* p) { return *reinterpret_cast<const uint4*>(p); }

template <int MODE, int NB, int KW, int U>
__global__ void __launch_bounds__(KW * 64) k_skinny(SkinnyArgs a) {
  constexpr int RT = ModeTraits<MODE>::RT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int wg = blockIdx.x;

  // ---- which weight rows this workgroup owns --------------------------------------
  const unsigned short* wrow[RT];
  int row0[RT];
  int which = 0, hl = 0, pidx = 0;  // QKV bookkeeping
  if (MODE == MODE_QKV) {
    const int half = a.d >> 1, pph = half >> 4;
    int head = wg / pph;
    pidx = wg - head * pph;
    const unsigned short* W;
    if (head < a.n_q) {
      which = 0; hl = head; W = a.w0;
    } else if (head < a.n_q + a.n_kv) {
      which = 1; hl = head - a.n_q; W = a.w1;
    } else {
      which = 2; hl = head - a.n_q - a.n_kv; W = a.w2;
    }
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      row0[t] = hl * a.d + t * half + pidx * 16;
      wrow[t] = W + (size_t)(row0[t] + i16) * a.K;
    }
  } else if (MODE == MODE_GATEUP) {
    row0[0] = wg * 16;
    int r = min(row0[0] + i16, a.n_rows - 1);
    wrow[0] = a.w0 + (size_t)r * a.K;
    if (RT > 1) {
      row0[RT - 1] = wg * 16;
      wrow[RT - 1] = a.w1 + (size_t)r * a.K;
    }
  } else {
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      row0[t] = (wg * RT + t) * 16;
      int r = min(row0[t] + i16, a.n_rows - 1);
      wrow[t] = a.w0 + (size_t)r * a.K;
    }
  }

  // ---- K range of this wave ----------------------------------------------------------
  const int steps = (a.K + 31) >> 5;
  const int s_begin = (int)(((long long)steps * wave) / KW), s_end = (int)(((long long)steps * (wave + 1)) / KW);

  const unsigned short* xrow[NB];
  bool xok[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    int jb = a.b0 + nb * 16 + i16;
    xok[nb] = jb < a.B;
    xrow[nb] = a.x + (size_t)(xok[nb] ? jb : a.b0) * a.K;
  }

  f32x4 acc[RT][NB];
#pragma unroll
  for (int t = 0; t < RT; ++t)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[t][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  for (int s = s_begin; s < s_end; s += U) {
    uint4 wf[U][RT], xf[U][NB];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = ((s + u) << 5) + g * 8;
      const bool ok = (s + u < s_end) && (k < a.K);
#pragma unroll
      for (int t = 0; t < RT; ++t) wf[u][t] = ok ? ld16(wrow[t] + k) : zero4;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) xf[u][nb] = (ok && xok[nb]) ? ld16(xrow[nb] + k) : zero4;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[t][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[u][t]),
                                                               __builtin_bit_cast(bf16x8, xf[u][nb]), acc[t][nb], 0, 0, 0);
  }

  // ---- reduce the K split through LDS ---------------------------------------------------
  __shared__ float4 red[KW][RT][NB][64];
#pragma unroll
  for (int t = 0; t < RT; ++t)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      red[wave][t][nb][lane] = make_float4(acc[t][nb][0], acc[t][nb][1], acc[t][nb][2], acc[t][nb][3]);
  __syncthreads();

  for (int nb = wave; nb < NB; nb += KW) {
    float v[RT][4];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      float4 sacc = red[0][t][nb][lane];
#pragma unroll
      for (int w = 1; w < KW; ++w) {
        float4 o = red[w][t][nb][lane];
        sacc.x += o.x; sacc.y += o.y; sacc.z += o.z; sacc.w += o.w;
      }
      v[t][0] = sacc.x; v[t][1] = sacc.y; v[t][2] = sacc.z; v[t][3] = sacc.w;
    }
    // this lane holds output rows row0 + 4g + {0..3} of batch entry jb
    const int jb = a.b0 + nb * 16 + i16;
    const bool active = jb < a.B;
    float rho = 1.f;
    if (MODE != MODE_RESID && active) rho = rsqrtf(a.ssq_in[jb] * a.inv_dim + a.eps);

    if (MODE == MODE_QKV) {
      if (!active) continue;
      const int half = a.d >> 1;
      const int idx0 = pidx * 16 + 4 * g;  // rotation index of v[.][0]
      float r0[4], r1[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a0 = v[0][e] * rho, a1 = v[1][e] * rho;
        if (which != 2) {
          const float2 cs = *reinterpret_cast<const float2*>(a.rope + ((size_t)jb * half + idx0 + e) * 2);
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
        const int n = a.kv_len[jb];
        const int lp = n / a.geom.page_tokens, slot = n - lp * a.geom.page_tokens;
        const int page = (n >= 0 && lp < a.max_pages) ? a.page_table[(size_t)jb * a.max_pages + lp] : -1;
        if (page < 0 || page >= a.geom.n_pages_total) {
          if (g == 0) atomicOr(a.err_flag, 1);
          continue;
        }
        // inside a page the order is [kv head][token slot][head_dim]
        char* base = a.slab + kv_page_off(a.geom, page, a.layer, which - 1) +
                     ((size_t)(hl * a.geom.page_tokens + slot) * a.d) * sizeof(unsigned short);
        unsigned short* dst = reinterpret_cast<unsigned short*>(base) + idx0;
        *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf2(r0[0], r0[1]), pack_bf2(r0[2], r0[3]));
        *reinterpret_cast<uint2*>(dst + half) = make_uint2(pack_bf2(r1[0], r1[1]), pack_bf2(r1[2], r1[3]));
      }
    } else if (MODE == MODE_RESID) {
      const int n0 = row0[0] + 4 * g;
      float s2 = 0.f;
      if (active) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = 0.f;
          if (n0 + e < a.n_rows) {
            o[e] = a.res[(size_t)jb * a.n_rows + n0 + e] + v[0][e];
            a.out[(size_t)jb * a.n_rows + n0 + e] = o[e];
            if (a.hxn) a.hxn[(size_t)jb * a.n_rows + n0 + e] = f2bf(o[e] * a.gnext[n0 + e]);
            s2 += o[e] * o[e];
          }
        }
      }
      s2 += __shfl_xor(s2, 16, 64);
      s2 += __shfl_xor(s2, 32, 64);
      if (active && g == 0 && a.ssq_out) atomicAdd(a.ssq_out + jb, s2);
    } else if (MODE == MODE_GATEUP) {
      if (!active) continue;
      const int n0 = row0[0] + 4 * g;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (n0 + e < a.n_rows) {
          float ga = v[0][e] * rho, up = v[1][e] * rho;
          float m = ga / (1.f + __expf(-ga)) * up;
          a.mbuf[(size_t)jb * a.n_rows + n0 + e] = f2bf(m);
        }
      }
    } else {  // MODE_LM
      if (!active) continue;
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        const int n0 = row0[t] + 4 * g;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n0 + e < a.n_rows) a.logits[(size_t)jb * a.n_rows + n0 + e] = v[t][e] * rho;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Step preparation: operand and sum of squares of the first layer, rotary table, cleared
// accumulators.  One workgroup per sequence.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_decode_prep(int H, int d, int n_ssq, int bpad, const int* token_ids,
                                                     const unsigned short* emb, int vocab, const float* x_in, float* xa,
                                                     const float* g1, unsigned short* hx1, float* ssq, float* rope,
                                                     const int* kv_len, float rope_base, int* err_flag) {
  const int b = blockIdx.x, tid = threadIdx.x;
  float s2 = 0.f;
  int tok = 0;
  if (token_ids) {
    tok = token_ids[b];
    if (tok < 0 || tok >= vocab) {
      if (tid == 0) atomicOr(err_flag, 2);
      tok = 0;
    }
  }
  for (int k = tid; k < H; k += 256) {
    float v = token_ids ? bf2f(emb[(size_t)tok * H + k]) : x_in[(size_t)b * H + k];
    if (token_ids) xa[(size_t)b * H + k] = v;
    hx1[(size_t)b * H + k] = f2bf(v * g1[k]);
    s2 += v * v;
  }
  __shared__ float sh[4];
  s2 = wave_sum(s2);
  if ((tid & 63) == 0) sh[tid >> 6] = s2;
  __syncthreads();
  if (tid == 0) ssq[b] = sh[0] + sh[1] + sh[2] + sh[3];
  for (int i = 1 + tid; i < n_ssq; i += 256) ssq[(size_t)i * bpad + b] = 0.f;
  const int half = d >> 1;
  const double pos = (double)kv_len[b];
  for (int i = tid; i < half; i += 256) {
    double theta = exp(-2.0 * (double)i / (double)d * log((double)rope_base));
    double ang = pos * theta;
    rope[((size_t)b * half + i) * 2 + 0] = (float)cos(ang);
    rope[((size_t)b * half + i) * 2 + 1] = (float)sin(ang);
  }
}

// ---------------------------------------------------------------------------------------------
// Paged attention for one new token per sequence (the bs*seqlen term of the paper's Eq. 1).
// Workgroup = (256-token chunk, KV head, sequence); each wave takes 4 pages of 16 tokens,
// issues all its K and V loads up front (16 B per lane, a page of one head is 4 KiB
// contiguous), takes the dot products on the vector ALUs with wavefront shuffles, and the
// workgroup merges its waves in LDS.  Sequences longer than one chunk write
// (max, sum, unnormalised output) partials; the last workgroup to arrive merges them.
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ void __launch_bounds__(256) k_paged_attn(const float* qbuf, const int* kv_len, const int* page_table,
                                                    int max_pages, int layer, int n_q, int n_kv, const char* slab,
                                                    KvGeom geom, float* part, int* cnt, int max_chunks,
                                                    unsigned short* obuf, int* err_flag) {
  constexpr int LPT = D / 8;         // lanes per token
  constexpr int TPI = 64 / LPT;      // tokens per load instruction
  constexpr int IT = kPageTokens / TPI;
  constexpr int PW = kChunkTokens / kPageTokens / 4;  // pages per wave
  const int b = blockIdx.z, c = blockIdx.y, ch = blockIdx.x;
  const int n_tot = kv_len[b] + 1;
  if (ch * kChunkTokens >= n_tot) return;
  const int nch = (n_tot + kChunkTokens - 1) / kChunkTokens;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int dg = lane % LPT, tl = lane / LPT;
  const int QD = n_q * D;

  uint4 kf[PW][IT], vf[PW][IT];
  bool ok[PW][IT];
#pragma unroll
  for (int pp = 0; pp < PW; ++pp) {
    const int lp = ch * (kChunkTokens / kPageTokens) + wave * PW + pp;
    const int tb = lp * kPageTokens;
    int page = -1;
    if (tb < n_tot && lp < max_pages) {
      page = page_table[(size_t)b * max_pages + lp];
      if (page < 0 || page >= geom.n_pages_total) {
        if (lane == 0) atomicOr(err_flag, 1);
        page = -1;
      }
    }
    const size_t offk = page >= 0 ? kv_page_off(geom, page, layer, 0) : 0;
    const size_t offv = page >= 0 ? kv_page_off(geom, page, layer, 1) : 0;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int slot = it * TPI + tl;
      ok[pp][it] = page >= 0 && (tb + slot) < n_tot;
      const size_t eo = ((size_t)(c * kPageTokens + slot) * D + dg * 8) * sizeof(unsigned short);
      kf[pp][it] = ok[pp][it] ? *reinterpret_cast<const uint4*>(slab + offk + eo) : make_uint4(0, 0, 0, 0);
      vf[pp][it] = ok[pp][it] ? *reinterpret_cast<const uint4*>(slab + offv + eo) : make_uint4(0, 0, 0, 0);
    }
  }

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
#pragma unroll
        for (int o = 1; o < LPT; o <<= 1) s += __shfl_xor(s, o, 64);
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
        const float p = ok[pp][it] ? exp2f(sc[gq][pp][it] - mw[gq]) : 0.f;
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
  __shared__ int s_last;
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
  for (int idx = tid; idx < G * D; idx += 256) {
    const int gq = idx / D, e = idx - gq * D;
    float M = fmaxf(fmaxf(s_m[0][gq], s_m[1][gq]), fmaxf(s_m[2][gq], s_m[3][gq]));
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = (s_m[w][gq] == -INFINITY) ? 0.f : exp2f(s_m[w][gq] - M);
      L += s_l[w][gq] * f;
      o += s_o[w][gq][e] * f;
    }
    const int head = c * G + gq;
    if (nch == 1) {
      obuf[(size_t)b * QD + head * D + e] = f2bf(o / L);
    } else {
      float* p = part + (((size_t)b * n_q + head) * max_chunks + ch) * (D + 2);
      p[2 + e] = o;
      if (e == 0) {
        p[0] = M;
        p[1] = L;
      }
    }
  }
  if (nch == 1) return;
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const int old = atomicAdd(cnt + b * n_kv + c, 1);
    s_last = (old == nch - 1);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int idx = tid; idx < G * D; idx += 256) {
    const int gq = idx / D, e = idx - gq * D;
    const int head = c * G + gq;
    const float* p = part + (((size_t)b * n_q + head) * max_chunks) * (D + 2);
    float M = -INFINITY;
    for (int i = 0; i < nch; ++i) M = fmaxf(M, __builtin_nontemporal_load(p + (size_t)i * (D + 2)));
    float L = 0.f, o = 0.f;
    for (int i = 0; i < nch; ++i) {
      const float f = exp2f(__builtin_nontemporal_load(p + (size_t)i * (D + 2)) - M);
      L += __builtin_nontemporal_load(p + (size_t)i * (D + 2) + 1) * f;
      o += __builtin_nontemporal_load(p + (size_t)i * (D + 2) + 2 + e) * f;
    }
    obuf[(size_t)b * QD + head * D + e] = f2bf(o / L);
  }
  if (tid == 0) cnt[b * n_kv + c] = 0;  // ready for the next step
}

__global__ void __launch_bounds__(256) k_argmax(const float* logits, int V, int* next_token) {
  const int b = blockIdx.x, tid = threadIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = tid; i < V; i += 256) {
    float v = logits[(size_t)b * V + i];
    if (v > best) {  // strided scan visits indices in increasing order per thread: first maximum is kept
      best = v;
      bi = i;
    }
  }
  __shared__ float sv[256];
  __shared__ int si[256];
  sv[tid] = best;
  si[tid] = bi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      if (sv[tid + s] > sv[tid] || (sv[tid + s] == sv[tid] && si[tid + s] < si[tid])) {
        sv[tid] = sv[tid + s];
        si[tid] = si[tid + s];
      }
    }
    __syncthreads();
  }
  if (tid == 0) next_token[b] = si[0];
}

template <int MODE, int NB, int KW, int U>
void launch_skinny(const SkinnyArgs& a, int n_wg, hipStream_t st) {
  hipLaunchKernelGGL((k_skinny<MODE, NB, KW, U>), dim3(n_wg), dim3(KW * 64), 0, st, a);
}

template <int MODE>
void dispatch_skinny(SkinnyArgs a, int n_wg, int kw8, hipStream_t st) {
  // passes of at most 64 batch rows; NB = 16-row tiles per pass
  for (int b0 = 0; b0 < a.B; b0 += 64) {
    a.b0 = b0;
    const int nb = (min(a.B - b0, 64) + 15) / 16;
    if (nb == 1) {
      if (kw8)
        launch_skinny<MODE, 1, 8, 8>(a, n_wg, st);
      else
        launch_skinny<MODE, 1, 4, 4>(a, n_wg, st);
    } else if (nb == 2) {
      launch_skinny<MODE, 2, 4, 4>(a, n_wg, st);
    } else {
      launch_skinny<MODE, 4, 4, 2>(a, n_wg, st);
    }
  }
}

}  // namespace

namespace harli {
harli_status decode_step_f32(harli_ctx* c, const harli_decode_batch* b, hipStream_t st);  // decode_generic.hip
}

extern "C" harli_status harli_decode_step(harli_ctx* c, const harli_decode_batch* b, void* hip_stream) {
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
  if (b->max_kv_len < 1 || b->max_kv_len > c->dw.max_chunks * kChunkTokens)
    return fail(HARLI_ERR_INVALID, "decode_step: max_kv_len %d outside 1..%d", b->max_kv_len,
                c->dw.max_chunks * kChunkTokens);
  if ((long long)b->max_pages * c->geom.page_tokens < b->max_kv_len)
    return fail(HARLI_ERR_INVALID, "decode_step: page table rows of %d pages cannot hold %d tokens", b->max_pages,
                b->max_kv_len);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (m.dtype == HARLI_F32) return decode_step_f32(c, b, st);

  DecodeWs& w = c->dw;
  const int B = b->batch, H = m.hidden, d = m.head_dim, QD = m.n_q_heads * d, F = m.ffn, L = m.n_layers;
  const int n_ssq = 2 * L + 1;
  hipLaunchKernelGGL(k_decode_prep, dim3(B), dim3(256), 0, st, H, d, n_ssq, w.bpad, b->token_ids,
                     static_cast<const unsigned short*>(c->emb), m.vocab, b->x_in, w.xa, c->layers[0].g1,
                     static_cast<unsigned short*>(w.hx1), w.ssq, w.rope, b->kv_len, m.rope_base, w.err_flag);

  const float* xcur = b->token_ids ? w.xa : b->x_in;
  float* ping[2] = {w.xb, w.xa};  // layer l writes ping[l&1]; layer 0 may not overwrite xa (it can be the input)
  const int n_chunks = (b->max_kv_len + kChunkTokens - 1) / kChunkTokens;
  const int G = m.n_q_heads / m.n_kv_heads;

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
    a.w0 = static_cast<const unsigned short*>(lw.w[0]);
    a.w1 = static_cast<const unsigned short*>(lw.w[1]);
    a.w2 = static_cast<const unsigned short*>(lw.w[2]);
    a.ssq_in = w.ssq + (size_t)(2 * l) * w.bpad;
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
    dispatch_skinny<MODE_QKV>(a, (m.n_q_heads + 2 * m.n_kv_heads) * (d / 32), 0, st);
    // --- attention
    {
      dim3 grid(n_chunks, m.n_kv_heads, B);
#define HARLI_ATTN(DD, GG)                                                                                         \
  hipLaunchKernelGGL((k_paged_attn<DD, GG>), grid, dim3(256), 0, st, w.qbuf, b->kv_len, b->page_table, b->max_pages, \
                     l, m.n_q_heads, m.n_kv_heads, c->slab, c->geom, w.att_part, w.att_cnt, w.max_chunks,             \
                     static_cast<unsigned short*>(w.obuf), w.err_flag)
      if (d == 128 && G == 1) HARLI_ATTN(128, 1);
      else if (d == 128 && G == 2) HARLI_ATTN(128, 2);
      else if (d == 128 && G == 4) HARLI_ATTN(128, 4);
      else if (d == 128 && G == 8) HARLI_ATTN(128, 8);
      else if (d == 64 && G == 1) HARLI_ATTN(64, 1);
      else if (d == 64 && G == 2) HARLI_ATTN(64, 2);
      else if (d == 64 && G == 4) HARLI_ATTN(64, 4);
      else return fail(HARLI_ERR_INVALID, "decode_step: head_dim %d with group %d is not supported", d, G);
#undef HARLI_ATTN
    }
    // --- output projection + residual, operand of the FFN
    a.x = static_cast<const unsigned short*>(w.obuf);
    a.K = QD;
    a.n_rows = H;
    a.w0 = static_cast<const unsigned short*>(lw.w[3]);
    a.res = xcur;
    a.out = w.x1;
    a.gnext = lw.g2;
    a.hxn = static_cast<unsigned short*>(w.hx2);
    a.ssq_out = w.ssq + (size_t)(2 * l + 1) * w.bpad;
    dispatch_skinny<MODE_RESID>(a, (H + 15) / 16, 1, st);
    // --- gate/up + SwiGLU
    a.x = static_cast<const unsigned short*>(w.hx2);
    a.K = H;
    a.n_rows = F;
    a.w0 = static_cast<const unsigned short*>(lw.w[4]);
    a.w1 = static_cast<const unsigned short*>(lw.w[5]);
    a.ssq_in = w.ssq + (size_t)(2 * l + 1) * w.bpad;
    a.mbuf = static_cast<unsigned short*>(w.mbuf);
    dispatch_skinny<MODE_GATEUP>(a, (F + 15) / 16, 0, st);
    // --- down projection + residual, operand of the next layer (or of the output layer)
    const bool last = (l == L - 1);
    float* xnext = (last && b->x_out) ? b->x_out : ping[l & 1];
    a.x = static_cast<const unsigned short*>(w.mbuf);
    a.K = F;
    a.n_rows = H;
    a.w0 = static_cast<const unsigned short*>(lw.w[6]);
    a.res = w.x1;
    a.out = xnext;
    a.gnext = last ? c->g_final : c->layers[l + 1].g1;
    a.hxn = (last && !b->logits) ? nullptr : static_cast<unsigned short*>(w.hx1);
    a.ssq_out = w.ssq + (size_t)(2 * l + 2) * w.bpad;
    dispatch_skinny<MODE_RESID>(a, (H + 15) / 16, 1, st);
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
    a.w0 = static_cast<const unsigned short*>(c->w_lm);
    a.ssq_in = w.ssq + (size_t)(2 * L) * w.bpad;
    a.logits = b->logits;
    dispatch_skinny<MODE_LM>(a, (m.vocab + 31) / 32, 0, st);
    if (b->next_token) hipLaunchKernelGGL(k_argmax, dim3(B), dim3(256), 0, st, b->logits, m.vocab, b->next_token);
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}
