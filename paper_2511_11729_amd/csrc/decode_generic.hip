// fp32-storage decode step (Harli Sec. 2.1 decode, Sec. 4.1 index-based KV): the same seven steps as the bf16
// path with every tensor -- weights, KV cache, activations -- held and computed in fp32.  This path serves
// small models and exact checks; it is written for any shape (no tile-size restrictions) with plain
// one-wave-per-output-row kernels and makes no use of the pre-shuffled weight copies.
#include "ctx.h"
#include "device_utils.h"

namespace harli {
namespace {

constexpr int kBT = 8;  // batch rows a wave carries per weight row

// x[b] = emb[token[b]] or x_in[b]
__global__ void __launch_bounds__(256) g_input(int H, const int* token_ids, const float* emb, int vocab, const float* x_in,
                                               float* x, int* err_flag) {
  const int b = blockIdx.x;
  const float* src;
  if (token_ids) {
    int t = token_ids[b];
    if (t < 0 || t >= vocab) {
      if (threadIdx.x == 0) atomicOr(err_flag, 2);
      t = 0;
    }
    src = emb + (size_t)t * H;
  } else {
    src = x_in + (size_t)b * H;
  }
  for (int i = threadIdx.x; i < H; i += 256) x[(size_t)b * H + i] = src[i];
}

// h[b] = x[b] * rsqrt(mean x^2 + eps) * g
__global__ void __launch_bounds__(256) g_rmsnorm(const float* x, const float* g, float* h, int H, float eps) {
  __shared__ float part[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  float s = 0.f;
  for (int i = tid; i < H; i += 256) {
    const float v = x[(size_t)b * H + i];
    s += v * v;
  }
  s = wave_sum(s);
  if ((tid & 63) == 0) part[tid >> 6] = s;
  __syncthreads();
  const float rho = rsqrtf((part[0] + part[1] + part[2] + part[3]) / (float)H + eps);
  for (int i = tid; i < H; i += 256) h[(size_t)b * H + i] = x[(size_t)b * H + i] * rho * g[i];
}

// y[b][n] = sum_k h[b][k] W[n][k] (+ res[b][n]); one wave per weight row n and tile of kBT batch rows
__global__ void __launch_bounds__(256) g_linear(const float* h, const float* W, const float* res, float* y, int B, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int b0 = blockIdx.y * kBT;
  if (n >= N) return;
  float acc[kBT];
#pragma unroll
  for (int i = 0; i < kBT; ++i) acc[i] = 0.f;
  const float* wr = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = wr[k];
#pragma unroll
    for (int i = 0; i < kBT; ++i) {
      const int b = min(b0 + i, B - 1);
      acc[i] += wv * h[(size_t)b * K + k];
    }
  }
#pragma unroll
  for (int i = 0; i < kBT; ++i) {
    const float s = wave_sum(acc[i]);
    if (lane == 0 && b0 + i < B) {
      const size_t o = (size_t)(b0 + i) * N + n;
      y[o] = s + (res ? res[o] : 0.f);
    }
  }
}

// rotary embedding of q (in place) and k at position kv_len[b]; k and v appended to the page of that position.
// One workgroup per sequence; pair (i, i + d/2) of every head, angle pos * base^(-2i/d) evaluated in double.
__global__ void __launch_bounds__(256) g_rope_append(float* q, const float* k, const float* v, const float* bq, const float* bk,
                                                     const float* bv, const int* kv_len,
                                                     const int* page_table, int max_pages, int layer, int n_q, int n_kv,
                                                     int d, const double* inv_freq, char* slab, KvGeom geom, int* err_flag) {
  const int b = blockIdx.x, tid = threadIdx.x, half = d / 2;
  const int pos = kv_len[b];
  const int lp = pos / geom.page_tokens, slot = pos - lp * geom.page_tokens;
  int page = (lp < max_pages) ? page_table[(size_t)b * max_pages + lp] : -1;
  const bool pgok = page >= 0 && page < geom.n_pages_total;
  if (!pgok && tid == 0) atomicOr(err_flag, 1);
  for (int idx = tid; idx < n_q * half; idx += 256) {
    const int hd = idx / half, i = idx - hd * half;
    const double ang = (double)pos * inv_freq[i];
    const float cs = (float)cos(ang), sn = (float)sin(ang);
    float* p = q + ((size_t)b * n_q + hd) * d;
    float a = p[i], c = p[i + half];
    if (bq) a += bq[hd * d + i], c += bq[hd * d + i + half];  // the bias precedes the rotation
    p[i] = a * cs - c * sn;
    p[i + half] = c * cs + a * sn;
  }
  if (!pgok) return;
  // inside a page the order is [kv head][token slot][head_dim]
  float* kp = reinterpret_cast<float*>(slab + kv_page_off(geom, page, layer, 0));
  float* vp = reinterpret_cast<float*>(slab + kv_page_off(geom, page, layer, 1));
  for (int idx = tid; idx < n_kv * half; idx += 256) {
    const int hd = idx / half, i = idx - hd * half;
    const double ang = (double)pos * inv_freq[i];
    const float cs = (float)cos(ang), sn = (float)sin(ang);
    const float* p = k + ((size_t)b * n_kv + hd) * d;
    float a = p[i], c = p[i + half];
    if (bk) a += bk[hd * d + i], c += bk[hd * d + i + half];
    const size_t o = ((size_t)hd * geom.page_tokens + slot) * d;
    kp[o + i] = a * cs - c * sn;
    kp[o + i + half] = c * cs + a * sn;
    const float* pv = v + ((size_t)b * n_kv + hd) * d;
    vp[o + i] = pv[i] + (bv ? bv[hd * d + i] : 0.f);
    vp[o + i + half] = pv[i + half] + (bv ? bv[hd * d + i + half] : 0.f);
  }
}

// attention of one (sequence, query head) over positions 0..kv_len[b]: scores to a scratch row, softmax, then P.V
__global__ void __launch_bounds__(256) g_attention(const float* q, const int* kv_len, const int* page_table, int max_pages,
                                                   int layer, int n_q, int n_kv, int d, const char* slab, KvGeom geom,
                                                   float* scores, int max_seq_len, float* o, int* err_flag) {
  __shared__ float red[4];
  __shared__ float bc;
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hk = hq / (n_q / n_kv);
  const int n_tot = min(min(kv_len[b] + 1, max_seq_len), max_pages * geom.page_tokens);
  if (n_tot != kv_len[b] + 1 && threadIdx.x == 0) atomicOr(err_flag, 4);  // the sequence is longer than the step was sized for
  const float* qv = q + ((size_t)b * n_q + hq) * d;
  float* sc = scores + ((size_t)b * n_q + hq) * max_seq_len;
  const float scale = rsqrtf((float)d);
  // scores: one wave per token
  for (int t = wave; t < n_tot; t += 4) {
    const int lp = t / geom.page_tokens, slot = t - lp * geom.page_tokens;
    const int page = page_table[(size_t)b * max_pages + lp];
    float s = 0.f;
    if (page >= 0 && page < geom.n_pages_total) {
      const float* kp = reinterpret_cast<const float*>(slab + kv_page_off(geom, page, layer, 0)) +
                        ((size_t)hk * geom.page_tokens + slot) * d;
      for (int e = lane; e < d; e += 64) s += qv[e] * kp[e];
    } else if (lane == 0) {
      atomicOr(err_flag, 1);
    }
    s = wave_sum(s);
    if (lane == 0) sc[t] = s * scale;
  }
  __syncthreads();
  float mx = -INFINITY;
  for (int t = tid; t < n_tot; t += 256) mx = fmaxf(mx, sc[t]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int t = tid; t < n_tot; t += 256) {
    const float p = expf(sc[t] - mx);
    sc[t] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) bc = 1.f / (red[0] + red[1] + red[2] + red[3]);
  __syncthreads();
  const float inv = bc;
  // o[e] = sum_t p[t] V[t][e]: thread per e
  for (int e = tid; e < d; e += 256) {
    float acc = 0.f;
    for (int t = 0; t < n_tot; ++t) {
      const int lp = t / geom.page_tokens, slot = t - lp * geom.page_tokens;
      const int page = page_table[(size_t)b * max_pages + lp];
      if (page < 0 || page >= geom.n_pages_total) continue;
      const float* vp = reinterpret_cast<const float*>(slab + kv_page_off(geom, page, layer, 1)) +
                        ((size_t)hk * geom.page_tokens + slot) * d;
      acc += sc[t] * vp[e];
    }
    o[((size_t)b * n_q + hq) * d + e] = acc * inv;
  }
}

// m = silu(a) * u
__global__ void __launch_bounds__(256) g_swiglu(const float* a, const float* u, float* m, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float av = a[i];
  m[i] = av / (1.f + expf(-av)) * u[i];
}

__global__ void __launch_bounds__(256) g_argmax(const float* logits, int V, int* next) {
  __shared__ float bv[256];
  __shared__ int bi[256];
  const int b = blockIdx.x, tid = threadIdx.x;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  for (int i = tid; i < V; i += 256) {
    const float v = logits[(size_t)b * V + i];
    if (v > best) best = v, idx = i;  // ascending i: the first maximum is kept
  }
  bv[tid] = best;
  bi[tid] = idx;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      if (bv[tid + s] > bv[tid] || (bv[tid + s] == bv[tid] && bi[tid + s] < bi[tid])) bv[tid] = bv[tid + s], bi[tid] = bi[tid + s];
    }
    __syncthreads();
  }
  if (tid == 0) next[b] = bi[0] == 0x7fffffff ? 0 : bi[0];
}

void linear(const float* h, const void* W, const float* res, float* y, int B, int N, int K, hipStream_t st) {
  hipLaunchKernelGGL(g_linear, dim3((N + 3) / 4, (B + kBT - 1) / kBT), dim3(256), 0, st, h, static_cast<const float*>(W), res, y,
                     B, N, K);
}

}  // namespace

harli_status decode_step_f32(harli_ctx* c, const harli_decode_batch* b, hipStream_t st) {
  const harli_model_cfg& m = c->cfg;
  DecodeWs& w = c->dw;
  const int B = b->batch, H = m.hidden, d = m.head_dim, QD = m.n_q_heads * d, KVD = m.n_kv_heads * d, F = m.ffn, L = m.n_layers;
  // fp32 views of the workspace (every operand buffer is allocated at 4 bytes per element)
  float* h = static_cast<float*>(w.hx1);     // normalised input of a projection
  float* o = static_cast<float*>(w.obuf);    // attention output
  float* q = w.qbuf;
  hipLaunchKernelGGL(g_input, dim3(B), dim3(256), 0, st, H, b->token_ids, static_cast<const float*>(c->emb), m.vocab, b->x_in,
                     w.xa, w.err_flag);
  float* x = w.xa;
  float* xn = w.xb;
  for (int l = 0; l < L; ++l) {
    const LayerDev& lw = c->layers[l];
    hipLaunchKernelGGL(g_rmsnorm, dim3(B), dim3(256), 0, st, x, lw.g1, h, H, m.rms_eps);
    linear(h, lw.w[0], nullptr, q, B, QD, H, st);
    linear(h, lw.w[1], nullptr, w.fk, B, KVD, H, st);
    linear(h, lw.w[2], nullptr, w.fv, B, KVD, H, st);
    hipLaunchKernelGGL(g_rope_append, dim3(B), dim3(256), 0, st, q, w.fk, w.fv, lw.bias[0], lw.bias[1], lw.bias[2], b->kv_len, b->page_table, b->max_pages, l,
                       m.n_q_heads, m.n_kv_heads, d, w.inv_freq, c->slab, c->geom, w.err_flag);
    hipLaunchKernelGGL(g_attention, dim3(m.n_q_heads, B), dim3(256), 0, st, q, b->kv_len, b->page_table, b->max_pages, l,
                       m.n_q_heads, m.n_kv_heads, d, c->slab, c->geom, w.scores, m.max_seq_len, o, w.err_flag);
    linear(o, lw.w[3], x, w.x1, B, H, QD, st);
    hipLaunchKernelGGL(g_rmsnorm, dim3(B), dim3(256), 0, st, w.x1, lw.g2, h, H, m.rms_eps);
    linear(h, lw.w[4], nullptr, w.fa, B, F, H, st);
    linear(h, lw.w[5], nullptr, w.fu, B, F, H, st);
    float* mm = static_cast<float*>(w.mbuf);
    const long long nf = (long long)B * F;
    hipLaunchKernelGGL(g_swiglu, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, st, w.fa, w.fu, mm, nf);
    const bool last = (l == L - 1);
    float* dst = (last && b->x_out) ? b->x_out : xn;
    linear(mm, lw.w[6], w.x1, dst, B, H, F, st);
    if (dst == xn) {
      float* t = x;
      x = xn;
      xn = t;
    } else {
      x = dst;
    }
  }
  if (b->logits) {
    hipLaunchKernelGGL(g_rmsnorm, dim3(B), dim3(256), 0, st, x, c->g_final, h, H, m.rms_eps);
    linear(h, c->w_lm, nullptr, b->logits, B, m.vocab, H, st);
    if (b->next_token) hipLaunchKernelGGL(g_argmax, dim3(B), dim3(256), 0, st, b->logits, m.vocab, b->next_token);
  }
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}

}  // namespace harli
