// LoRA finetune unit: one transformer layer x one micro-batch, forward and backward
// (Harli Sec. 6.1 scheduling unit; Sec. 2.1: base parameters frozen, only the adapters get
// gradients; Sec. 4: the activations kept for backward live in the unified pool).
//
// Forward  y = x W^T + s (x A) B  rides on one GEMM per projection: the adapter is a second K
// segment [s x A | B^T] of the base GEMM.  Backward needs no weight gradients for the frozen
// base: dx = dy W + (s dy B^T) A^T is again one multi-segment GEMM against a library-owned
// transposed copy of W, and dA = x^T (s dy B^T), dB = (s x A)^T dy are skinny reductions over
// the tokens (the adapters' contributions to dx ride on the backward GEMMs as further K
// segments).  Attention is the fused forward / dQ / dK-dV kernels of ft_attention.hip (head
// sizes 64 and 128; harli_lora_attach refuses any other).
#include <algorithm>
#include <cmath>
#include <vector>

#include "ctx.h"
#include "ft_elem.h"
#include "ft_attention.h"
#include "ft_kernels.h"
#include "gemm_timer.h"
#include "gemm2.h"
#include "window.h"

using namespace harli;

namespace harli {
harli_status pool_free_owned(harli_pool* p, const harli_alloc* a, void* event);  // pool.cpp
harli_status head_prepare(harli_ctx* c);                                          // head.hip
}

struct harli_saved {
  int layer = 0, Bf = 0, S = 0, T = 0;
  const float* X = nullptr;  // borrowed from the caller
  harli_alloc big{};
  std::vector<harli_alloc> small;
  float *rho1 = nullptr, *rho2 = nullptr, *lse = nullptr, *x1 = nullptr;
  bf *h = nullptr, *q = nullptr, *k = nullptr, *v = nullptr, *o = nullptr, *h2 = nullptr, *a = nullptr,
     *u = nullptr, *m = nullptr;
  bf* us[kTargets] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
};

namespace {

inline size_t al(size_t n) { return (n + 255) & ~size_t(255); }

// workspace carved from one device allocation
struct FtWs {
  size_t bytes = 0;
  char* base = nullptr;
  float *delta = nullptr, *dh2 = nullptr,
        *dx1 = nullptr, *dh = nullptr, *gpart = nullptr;
  bf *vT = nullptr, *At[kTargets] = {}, *Bt[kTargets] = {}, *dyb = nullptr, *da = nullptr, *du = nullptr, *dx1b = nullptr, *dob = nullptr,
     *doT = nullptr, *qT = nullptr, *kT = nullptr, *dq = nullptr, *dkq = nullptr,
     *dvq = nullptr, *dk = nullptr, *dv = nullptr, *gs[3] = {}, *An[kTargets] = {}, *Bn[kTargets] = {};
  float* scale = nullptr;  // [0] sigma, [1] 1/sigma, [2], [3] maxima of this and the next call: gradient scaling of the backward pass
  int scale_parity = 0;
  int Bf = 0, S = 0;
};

struct FtState {
  FtWs ws;
  bool ws_in_pool = false;   // ws.base is ws_alloc (a TENSOR allocation of the unified pool) rather than a library allocation
  harli_alloc ws_alloc{};
  size_t weight_bytes = 0;   // private copies of the frozen weights, biases and the ones column
};

FtState* state(harli_ctx* c) { return static_cast<FtState*>(c->ft_ws); }

// gives the workspace back (waits for the device first: units in flight may still use it)
harli_status free_ws(harli_ctx* c) {
  FtState* fs = state(c);
  if (!fs || !fs->ws.base) return HARLI_OK;
  HARLI_HIP(hipDeviceSynchronize());
  if (fs->ws_in_pool) {
    harli_status r = harli_pool_free(c->pool, &fs->ws_alloc, nullptr);
    if (r != HARLI_OK) return r;
  } else {
    HARLI_HIP(hipFree(fs->ws.base));
  }
  fs->ws.base = nullptr;
  fs->ws.bytes = 0;
  fs->ws_in_pool = false;
  return HARLI_OK;
}

struct Dims {
  int T, H, QD, KVD, F, d, nq, nkv, G, r, Z;
};

Dims dims(const harli_ctx* c, int Bf, int S) {
  const harli_model_cfg& m = c->cfg;
  Dims D;
  D.T = Bf * S;
  D.H = m.hidden;
  D.d = m.head_dim;
  D.nq = m.n_q_heads;
  D.nkv = m.n_kv_heads;
  D.QD = D.nq * D.d;
  D.KVD = D.nkv * D.d;
  D.F = m.ffn;
  D.G = D.nq / D.nkv;
  D.r = c->lora.rank;
  D.Z = Bf * D.nq;
  return D;
}

// The unit's workspace (backward temporaries, adapter copies, gradient scratch), sized once for max_ft_tokens when the
// adapters are attached, so that no forward or backward call allocates or frees device memory (either would be a
// device-wide synchronisation in the middle of serving).  With workspace_in_pool it is one TENSOR allocation of the
// unified pool (Sec. 4.2: every byte a task uses comes from the one pool, so the pool's statistics and its
// inference-first back-pressure, Sec. 4.4, see it); otherwise the library allocates it itself.
harli_status make_ws(harli_ctx* c) {
  FtState* fs = state(c);
  FtWs& w = fs->ws;
  const Dims D = dims(c, 1, c->cfg.max_ft_tokens);
  const size_t T = D.T;
  const size_t maxdim = std::max(std::max((size_t)D.H, (size_t)D.QD), (size_t)D.F);
  size_t off = 0;
  auto take = [&](size_t n) {
    size_t o = off;
    off += al(n);
    return o;
  };
  const size_t o_delta = take(T * D.nq * 4);
  const size_t o_dh2 = take(T * D.H * 4), o_dx1 = take(T * D.H * 4), o_dh = take(T * D.H * 4);
  const size_t o_vT = take(T * D.KVD * 2), o_kT = take(T * D.KVD * 2), o_qT = take(T * D.QD * 2), o_doT = take(T * D.QD * 2);
  const size_t ad = al(maxdim * D.r * 2);  // one adapter matrix in the compute element, row-major (skinny products)
  const size_t adb = al(blocked_elems((long long)maxdim, D.r) * 2);  // ... in the weight GEMM's blocked order
  const size_t o_At = take(kTargets * ad), o_Bt = take(kTargets * adb);
  const size_t o_An = take(kTargets * adb), o_Bn = take(kTargets * ad), o_scale = take(64);
  const size_t o_dyb = take(T * D.H * 2), o_da = take(T * D.F * 2), o_du = take(T * D.F * 2), o_dx1b = take(T * D.H * 2);
  const size_t o_dob = take(T * D.QD * 2), o_dq = take(T * D.QD * 2), o_dkq = take(T * D.QD * 2), o_dvq = take(T * D.QD * 2);
  const size_t o_dk = take(T * D.KVD * 2), o_dv = take(T * D.KVD * 2), o_gs = take(3 * al(T * D.r * 2));
  const size_t o_gpart = take(ft_lora_grad_ws_floats((int)maxdim, D.r) * 4);
  const bool want_pool = c->lora.workspace_in_pool != 0 || c->cfg.memory_in_pool != 0;
  if (off != w.bytes || want_pool != fs->ws_in_pool) {  // first attach, or another rank / placement than before
    harli_status r = free_ws(c);
    if (r != HARLI_OK) return r;
    if (want_pool) {
      r = harli_pool_alloc(c->pool, HARLI_CLS_TENSOR, off, &fs->ws_alloc);
      if (r != HARLI_OK) return r;
      w.base = static_cast<char*>(fs->ws_alloc.ptr);
    } else {
      HARLI_HIP(hipMalloc(reinterpret_cast<void**>(&w.base), off));
    }
    fs->ws_in_pool = want_pool;
    w.bytes = off;
  }
  char* b = w.base;
  w.delta = (float*)(b + o_delta);
  w.dh2 = (float*)(b + o_dh2); w.dx1 = (float*)(b + o_dx1); w.dh = (float*)(b + o_dh);
  w.vT = (bf*)(b + o_vT); w.kT = (bf*)(b + o_kT); w.qT = (bf*)(b + o_qT); w.doT = (bf*)(b + o_doT);
  w.dyb = (bf*)(b + o_dyb); w.da = (bf*)(b + o_da); w.du = (bf*)(b + o_du);
  w.dx1b = (bf*)(b + o_dx1b); w.dob = (bf*)(b + o_dob); w.dq = (bf*)(b + o_dq); w.dkq = (bf*)(b + o_dkq);
  w.dvq = (bf*)(b + o_dvq); w.dk = (bf*)(b + o_dk); w.dv = (bf*)(b + o_dv);
  for (int i = 0; i < 3; ++i) w.gs[i] = (bf*)(b + o_gs + i * al(T * D.r * 2));
  w.gpart = (float*)(b + o_gpart);
  for (int i = 0; i < kTargets; ++i) {
    w.At[i] = (bf*)(b + o_At + i * ad); w.Bt[i] = (bf*)(b + o_Bt + i * adb);
    w.An[i] = (bf*)(b + o_An + i * adb); w.Bn[i] = (bf*)(b + o_Bn + i * ad);
  }
  w.scale = (float*)(b + o_scale);
  HARLI_HIP(hipMemset(w.scale, 0, 64));  // the maxima start at zero; every backward call clears the slot of the next
  w.scale_parity = 0;
  return HARLI_OK;
}

// Per call: the workspace was sized at attach for max_ft_tokens; only the shape of the call is recorded.
harli_status ensure_ws(harli_ctx* c, int Bf, int S) {
  FtWs& w = state(c)->ws;
  w.Bf = Bf;
  w.S = S;
  return HARLI_OK;
}

inline bool adapted(const harli_ctx* c, int t) { return (c->lora.targets >> t) & 1u; }
inline float lscale(const harli_ctx* c) { return c->lora.alpha / (float)c->lora.rank; }

// Every adapted projection's A and B (storage type, contents may change between calls) converted to the compute
// element in two launches.  Forward: A^T [r, in] row-major for the skinny product s x A, and B^T as the weight GEMM's
// blocked operand [out rows, r].  Backward: B [r, out] row-major for s dy B^T, and A as the blocked operand [in rows, r].
void convert_adapters(harli_ctx* c, const LayerDev& L, bool forward, hipStream_t st) {
  FtWs& w = state(c)->ws;
  FtConvJobs jobs{};
  BlockJobs blk{};
  blk.half = 1;
  jobs.flag = blk.flag = c->dw.err_flag;
  for (int t = 0; t < kTargets; ++t) {
    if (!adapted(c, t)) continue;
    int out, in;
    proj_shape(c->cfg, t, &out, &in);
    const int r = c->lora.rank;
    const int f32 = c->cfg.dtype == HARLI_F32 ? 1 : 0;
    if (forward) {
      jobs.j[jobs.n++] = FtConvJob{L.A[t], w.At[t], in, r, 1, f32};
      blk.j[blk.n++] = BlockJob{L.B[t], w.Bt[t], r, out, 1, f32};  // operand [n = out][k = r] = B[k][n]
    } else {
      blk.j[blk.n++] = BlockJob{L.A[t], w.An[t], in, r, 0, f32};   // operand [n = in][k = r] = A[n][k]
      jobs.j[jobs.n++] = FtConvJob{L.B[t], w.Bn[t], r, out, 0, f32};
    }
  }
  if (jobs.n) ft_convert_jobs(jobs, st);
  gemm2_block_jobs(blk, st);
}

// forward of one projection: out = xin . W^T (+ us . Bt^T), us = s * xin . A kept for backward
// us_t = s * xin . A_t for every adapted projection t of a group that reads the same input, in one launch
void proj_us_group(harli_ctx* c, int t_first, int t_last, const bf* xin, int T, harli_saved* sv, hipStream_t st) {
  FtWs& w = state(c)->ws;
  const int r = c->lora.rank;
  SkinnyNtJobs jobs{};
  for (int t = t_first; t <= t_last; ++t) {
    if (!adapted(c, t)) continue;
    int out, in;
    proj_shape(c->cfg, t, &out, &in);
    // ws.At[t] = A^T [r, in] was made by convert_adapters at the top of the call
    jobs.j[jobs.n++] = SkinnyNtJob{xin, in, w.At[t], in, sv->us[t], r, r, in};
  }
  ft_skinny_nt_multi(jobs, T, lscale(c), c->dw.err_flag, st);
}

// ---- the weight GEMMs (gemm2.h) ----
inline int tiles256(int n) { return (n + kG2TileN - 1) / kG2TileN; }
Gemm2Args wg_begin(const harli_ctx* c, int T) {
  Gemm2Args g{};
  g.M = T;
  g.alpha = 1.f;
  g.half = 1;
  g.overflow_flag = c->dw.err_flag;
  return g;
}
void wg_seg(Gemm2Args& g, const bf* A, long long lda, int K, const void* B, int rows, int t0, int t1, const void* B2 = nullptr, int pair = 0) {
  Gemm2Seg& q = g.seg[g.nseg++];
  q = Gemm2Seg{};
  q.A = A;
  q.lda = lda;
  q.K = K;
  q.B = static_cast<const unsigned short*>(B);
  q.B2 = static_cast<const unsigned short*>(B2);
  q.pair = pair;
  q.rows = rows;
  q.tile0 = t0;
  q.tile1 = t1;
}
// one projection's segments over the output tiles [t0, t1): x W^T, the frozen bias (eight more contraction columns:
// ones on the input side, (b, 0, ..., 0) on the weight side) and the adapter s (x A) B (us_t made by proj_us_group)
void wg_proj(harli_ctx* c, Gemm2Args& g, const LayerDev& L, int t, const bf* xin, const harli_saved* sv, int t0, int t1) {
  int out, in;
  proj_shape(c->cfg, t, &out, &in);
  FtWs& w = state(c)->ws;
  wg_seg(g, xin, in, in, L.w16[t], out, t0, t1);
  if (t < 3 && L.b16[t]) wg_seg(g, static_cast<const bf*>(c->ones16), 8, 8, L.b16[t], out, t0, t1);
  if (adapted(c, t)) wg_seg(g, sv->us[t], c->lora.rank, c->lora.rank, w.Bt[t], out, t0, t1);
}
void wg_out_f32(Gemm2Args& g, float* Cf, const float* res, int N) {
  g.nout = 1;
  g.tiles_n = tiles256(N);
  g.out[0] = Gemm2Out{0, N, nullptr, 0, Cf, res, N};
}
void wg_out_16(Gemm2Args& g, bf* Cb, int N) {
  g.nout = 1;
  g.tiles_n = tiles256(N);
  g.out[0] = Gemm2Out{0, N, Cb, N, nullptr, nullptr, 0};
}

// adapter gradients of one projection given dy (bf16 [T, out]) and its input xin (bf16 [T, in]);
// leaves gs = s * dy . B^T in ws.gs[slot]: the caller adds (gs, ws.An[t])
// to its dx GEMM as one more K segment (dx += gs . A^T)
// One or more projections that read the same input xin: their 2 n gradient products go out as one pair of launches.
harli_status proj_grads_group(harli_ctx* c, int n, const int* ts, const int* slots, const bf* const* dys, const bf* xin, int T,
                              const harli_saved* sv, float* const* dA, float* const* dB, hipStream_t st) {
  FtWs& w = state(c)->ws;
  const int r = c->lora.rank;
  LoraGradJobs jobs{};
  SkinnyNtJobs sk{};
  for (int i = 0; i < n; ++i) {
    const int t = ts[i];
    int out, in;
    proj_shape(c->cfg, t, &out, &in);
    // ws.An[t] = A [in, r] and ws.Bn[t] = B [r, out] in the compute element were made by convert_adapters
    sk.j[sk.n++] = SkinnyNtJob{dys[i], out, w.Bn[t], out, w.gs[slots[i]], r, r, out};  // gs = s * dy . B^T   (carries sigma)
    jobs.j[jobs.n++] = LoraGradJob{xin, in, w.gs[slots[i]], r, dA[t], r, 1, in, 0, 0, 0, 0};      // dA += x^T gs / sigma
    jobs.j[jobs.n++] = LoraGradJob{dys[i], out, sv->us[t], r, dB[t], 1, out, out, 0, 0, 0, 0};    // dB += us^T dy / sigma
  }
  ft_skinny_nt_multi(sk, T, lscale(c), c->dw.err_flag, st);
  ft_lora_grad_multi(jobs, T, r, w.scale + 1, w.gpart, st);
  return HARLI_OK;
}
harli_status proj_grads(harli_ctx* c, const LayerDev& L, int t, int slot, const bf* dy, const bf* xin, int T,
                        const harli_saved* sv, float* const* dA, float* const* dB, hipStream_t st) {
  (void)L;
  return proj_grads_group(c, 1, &t, &slot, &dy, xin, T, sv, dA, dB, st);
}

harli_status check_call(harli_ctx* c, int layer, int Bf, int S, const char* who) {
  if (!c) return fail(HARLI_ERR_INVALID, "%s: null context", who);
  if (!c->lora_attached) return fail(HARLI_ERR_STATE, "%s: call harli_lora_attach first", who);
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(HARLI_ERR_INVALID, "%s: layer %d out of range", who, layer);
  if (Bf < 1 || S < 1 || (long long)Bf * S > c->cfg.max_ft_tokens)
    return fail(HARLI_ERR_INVALID, "%s: %d x %d tokens exceed max_ft_tokens %d", who, Bf, S, c->cfg.max_ft_tokens);
  if (S % 8) return fail(HARLI_ERR_INVALID, "%s: sequence length must be a multiple of 8", who);
  return HARLI_OK;
}

struct SavedPlan {
  size_t big_bytes;
  size_t o_x1, o_h, o_q, o_k, o_v, o_o, o_h2, o_a, o_u, o_m;
};

SavedPlan plan_saved(const harli_ctx* c, const Dims& D, int S) {
  SavedPlan p{};
  size_t off = 0;
  auto take = [&](size_t n) {
    size_t o = off;
    off += al(n);
    return o;
  };
  const size_t T = D.T;
  p.o_x1 = take(T * D.H * 4);
  p.o_h = take(T * D.H * 2);
  p.o_q = take(T * D.QD * 2);
  p.o_k = take(T * D.KVD * 2);
  p.o_v = take(T * D.KVD * 2);
  p.o_o = take(T * D.QD * 2);
  p.o_h2 = take(T * D.H * 2);
  p.o_a = take(T * D.F * 2);
  p.o_u = take(T * D.F * 2);
  p.o_m = take(T * D.F * 2);
  p.big_bytes = off;
  return p;
}

void release_saved(harli_ctx* c, harli_saved* sv, hipStream_t st, bool with_event) {
  auto rel = [&](const harli_alloc& a) {
    void* ev = nullptr;
    if (with_event) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess) {
        if (hipEventRecord(e, st) == hipSuccess)
          ev = e;
        else
          (void)hipEventDestroy(e);
      }
    }
    (void)pool_free_owned(c->pool, &a, ev);
  };
  if (sv->big.ptr) rel(sv->big);
  for (const harli_alloc& a : sv->small) rel(a);
  delete sv;
}

}  // namespace

namespace harli {
void free_finetune_state(harli_ctx* c) {
  for (LayerDev& L : c->layers)
    for (int t = 0; t < 3; ++t)
      if (L.b16[t]) {
        lib_free(c, L.b16[t]);
        L.b16[t] = nullptr;
      }
  if (c->ones16) {
    lib_free(c, c->ones16);
    c->ones16 = nullptr;
  }
  for (LayerDev& L : c->layers)
    for (int t = 0; t < kTargets; ++t)
      if (L.wt[t]) {
        lib_free(c, L.wt[t]);
        L.wt[t] = nullptr;
        lib_free(c, L.w16[t]);
        L.w16[t] = nullptr;
      }
  if (c->ft_ws) {
    FtState* s = state(c);
    (void)free_ws(c);
    delete s;
    c->ft_ws = nullptr;
  }
}
}  // namespace harli

extern "C" harli_status harli_lora_attach(harli_ctx* c, const harli_lora_cfg* cfg, void* const* A, void* const* B) {
  if (!c || !cfg || !A || !B) return fail(HARLI_ERR_INVALID, "lora_attach: null argument");
  if (cfg->rank != 8 && cfg->rank != 16 && cfg->rank != 32 && cfg->rank != 64)
    return fail(HARLI_ERR_INVALID, "lora_attach: rank must be 8, 16, 32 or 64, got %d", cfg->rank);
  if (cfg->targets == 0 || cfg->targets >= (1u << kTargets)) return fail(HARLI_ERR_INVALID, "lora_attach: bad target mask");
  if (cfg->grad_headroom_log2 < 0 || cfg->grad_headroom_log2 > 24)
    return fail(HARLI_ERR_INVALID, "lora_attach: grad_headroom_log2 %d outside 0..24", cfg->grad_headroom_log2);
  if (c->cfg.max_ft_tokens < 1) return fail(HARLI_ERR_STATE, "lora_attach: the context was created with max_ft_tokens = 0");
  if (!ft_attn_supported(c->cfg.head_dim))
    return fail(HARLI_ERR_INVALID, "lora_attach: the finetune attention kernels cover head_dim 64 and 128, got %d", c->cfg.head_dim);
  if (c->window) return fail(HARLI_ERR_STATE, "lora_attach: disable the weight window first");
  for (int l = 0; l < c->cfg.n_layers; ++l)
    for (int t = 0; t < kTargets; ++t)
      if (((cfg->targets >> t) & 1u) && (!A[l * kTargets + t] || !B[l * kTargets + t]))
        return fail(HARLI_ERR_INVALID, "lora_attach: layer %d target %d has a null adapter", l, t);
  c->lora = *cfg;
  c->lora_attached = false;  // until everything below has succeeded
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    LayerDev& L = c->layers[l];
    for (int t = 0; t < kTargets; ++t) {
      const bool on = (cfg->targets >> t) & 1u;
      L.A[t] = on ? A[l * kTargets + t] : nullptr;
      L.B[t] = on ? B[l * kTargets + t] : nullptr;
      if (!L.wt[t]) {  // finetune-private copies of the frozen weights in the compute element, in the weight GEMM's
        int out, in;   // blocked order: W as the operand [out rows, in] of the forward pass, W^T [in rows, out] for dx = dy W
        proj_shape(c->cfg, t, &out, &in);
        const size_t nb = ft_weight_copy_bytes(out, in);
        harli_status am = lib_alloc(c, &L.wt[t], nb);
        if (am == HARLI_OK) am = lib_alloc(c, &L.w16[t], nb);
        if (am != HARLI_OK) {  // a half-made pair would look attached to the next call
          lib_free(c, L.wt[t]);
          L.wt[t] = L.w16[t] = nullptr;
          return am;
        }
        const int f32 = c->cfg.dtype == HARLI_F32 ? 1 : 0;
        BlockJobs jobs{};
        jobs.half = 1;
        jobs.flag = c->dw.err_flag;
        jobs.j[jobs.n++] = BlockJob{L.w[t], static_cast<bf*>(L.w16[t]), out, in, 0, f32};
        jobs.j[jobs.n++] = BlockJob{L.w[t], static_cast<bf*>(L.wt[t]), out, in, 1, f32};
        gemm2_block_jobs(jobs, nullptr);
      }
    }
  }
  // biases of q, k, v in the compute element ([out, 8], bias in column 0) and the column of ones they multiply
  bool any_bias = false;
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    LayerDev& L = c->layers[l];
    for (int t = 0; t < 3; ++t) {
      if (!L.bias[t] || L.b16[t]) continue;
      any_bias = true;
      int out, in;
      proj_shape(c->cfg, t, &out, &in);
      std::vector<float> hb(out);
      HARLI_HIP(hipMemcpy(hb.data(), L.bias[t], (size_t)out * 4, hipMemcpyDeviceToHost));
      // blocked operand [out rows, K = 8]: one K step per row tile, row n of a tile at 32 n, the bias in column 0
      std::vector<unsigned short> h16(blocked_elems(out, 8), 0);
      for (int n = 0; n < out; ++n) h16[(size_t)(n / kG2TileN) * (kG2TileN * kG2StepK) + (size_t)(n % kG2TileN) * kG2StepK] = host_to_elem(hb[n]);
      {
        harli_status am = lib_alloc(c, &L.b16[t], h16.size() * 2);
        if (am != HARLI_OK) return am;
      }
      HARLI_HIP(hipMemcpy(L.b16[t], h16.data(), h16.size() * 2, hipMemcpyHostToDevice));
    }
  }
  if (any_bias && !c->ones16) {
    std::vector<unsigned short> ones((size_t)c->cfg.max_ft_tokens * 8, host_to_elem(1.0f));
    {
      harli_status am = lib_alloc(c, &c->ones16, ones.size() * 2);
      if (am != HARLI_OK) return am;
    }
    HARLI_HIP(hipMemcpy(c->ones16, ones.data(), ones.size() * 2, hipMemcpyHostToDevice));
  }
  HARLI_HIP(hipDeviceSynchronize());
  {  // a frozen weight that half cannot hold would be clamped in the private copies: refuse it here, by name
    int flag = 0;
    HARLI_HIP(hipMemcpy(&flag, c->dw.err_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (flag & 8) {
      flag &= ~8;
      HARLI_HIP(hipMemcpy(c->dw.err_flag, &flag, sizeof(int), hipMemcpyHostToDevice));
      for (LayerDev& L : c->layers)
        for (int t = 0; t < kTargets; ++t) {
          lib_free(c, L.wt[t]);
          lib_free(c, L.w16[t]);
          L.wt[t] = L.w16[t] = nullptr;
        }
      return fail(HARLI_ERR_INVALID, "lora_attach: a frozen weight lies beyond the range of the 16-bit compute element (|w| > 65504)");
    }
  }
  if (!c->ft_ws) c->ft_ws = new FtState;
  {
    size_t nb = 0;
    for (int l = 0; l < c->cfg.n_layers; ++l)
      for (int t = 0; t < kTargets; ++t) {
        int out, in;
        proj_shape(c->cfg, t, &out, &in);
        if (c->layers[l].wt[t]) nb += 2 * ft_weight_copy_bytes(out, in);
        if (t < 3 && c->layers[l].b16[t]) nb += blocked_elems(out, 8) * 2;
      }
    if (c->ones16) nb += (size_t)c->cfg.max_ft_tokens * 16;
    state(c)->weight_bytes = nb;
  }
  harli_status ws = make_ws(c);
  if (ws == HARLI_OK) ws = head_prepare(c);
  if (ws != HARLI_OK) return ws;
  c->lora_attached = true;
  return HARLI_OK;
}

namespace harli {
// device memory the finetune side holds: (private weight copies, workspace, whether the workspace is in the pool)
void finetune_device_bytes(const harli_ctx* c, size_t* weights, size_t* workspace, int* in_pool) {
  *weights = *workspace = 0;
  *in_pool = 0;
  if (!c->ft_ws) return;
  const FtState* fs = static_cast<const FtState*>(c->ft_ws);
  *weights = fs->weight_bytes;
  *workspace = fs->ws.bytes;
  *in_pool = fs->ws_in_pool ? 1 : 0;
}
}  // namespace harli

extern "C" harli_status harli_saved_bytes(const harli_ctx* c, int32_t B_f, int32_t S, size_t* bytes) {
  if (!c || !bytes || B_f < 1 || S < 1) return fail(HARLI_ERR_INVALID, "saved_bytes: bad argument");
  if (!c->lora_attached) return fail(HARLI_ERR_STATE, "saved_bytes: call harli_lora_attach first");
  const Dims D = dims(c, B_f, S);
  size_t n = plan_saved(c, D, S).big_bytes;
  n += 2 * (size_t)D.T * 4 + (size_t)D.Z * S * 4;
  for (int t = 0; t < kTargets; ++t)
    if (adapted(c, t)) n += (size_t)D.T * D.r * 2;
  *bytes = n;
  return HARLI_OK;
}

extern "C" harli_status harli_lora_fwd(harli_ctx* c, int32_t layer, const float* X, float* Y, int32_t B_f, int32_t S,
                                       harli_saved** saved, void* hip_stream) {
  harli_status s = check_call(c, layer, B_f, S, "lora_fwd");
  if (s != HARLI_OK) return s;
  if (!X || !Y || !saved) return fail(HARLI_ERR_INVALID, "lora_fwd: null argument");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const harli_model_cfg& m = c->cfg;
  const Dims D = dims(c, B_f, S);
  const LayerDev& L = c->layers[layer];
  s = ensure_ws(c, B_f, S);
  if (s != HARLI_OK) return s;
  FtWs& w = state(c)->ws;
  s = window_acquire(c, layer, false, st);
  if (s != HARLI_OK) return s;

  // ---- activations kept for backward come from the unified pool ----
  harli_saved* sv = new harli_saved;
  sv->layer = layer;
  sv->Bf = B_f;
  sv->S = S;
  sv->T = D.T;
  sv->X = X;
  const SavedPlan pl = plan_saved(c, D, S);
  s = harli_pool_alloc(c->pool, HARLI_CLS_AUTO, pl.big_bytes, &sv->big);
  if (s != HARLI_OK) {
    delete sv;
    return s;
  }
  auto small = [&](size_t n, void** p) -> harli_status {
    harli_alloc a{};
    harli_status r = harli_pool_alloc(c->pool, HARLI_CLS_AUTO, n, &a);
    if (r != HARLI_OK) return r;
    sv->small.push_back(a);
    *p = a.ptr;
    return HARLI_OK;
  };
  s = small((size_t)D.T * 4, reinterpret_cast<void**>(&sv->rho1));
  if (s == HARLI_OK) s = small((size_t)D.T * 4, reinterpret_cast<void**>(&sv->rho2));
  if (s == HARLI_OK) s = small((size_t)D.Z * S * 4, reinterpret_cast<void**>(&sv->lse));
  for (int t = 0; t < kTargets && s == HARLI_OK; ++t)
    if (adapted(c, t)) s = small((size_t)D.T * D.r * 2, reinterpret_cast<void**>(&sv->us[t]));
  if (s != HARLI_OK) {
    release_saved(c, sv, st, false);  // nothing was launched on these buffers
    return s;
  }
  char* bb = static_cast<char*>(sv->big.ptr);
  sv->x1 = (float*)(bb + pl.o_x1); sv->h = (bf*)(bb + pl.o_h); sv->q = (bf*)(bb + pl.o_q); sv->k = (bf*)(bb + pl.o_k);
  sv->v = (bf*)(bb + pl.o_v); sv->o = (bf*)(bb + pl.o_o); sv->h2 = (bf*)(bb + pl.o_h2);
  sv->a = (bf*)(bb + pl.o_a); sv->u = (bf*)(bb + pl.o_u); sv->m = (bf*)(bb + pl.o_m);

#define RUN(x)                          \
  do {                                  \
    harli_status r_ = (x);              \
    if (r_ != HARLI_OK) {               \
      release_saved(c, sv, st, true);   \
      return r_;                        \
    }                                   \
  } while (0)

  const int T = D.T;
  convert_adapters(c, L, true, st);
  ft_rmsnorm_fwd(X, L.g1, sv->h, sv->rho1, T, D.H, m.rms_eps, c->dw.err_flag, st);
  proj_us_group(c, 0, 2, sv->h, T, sv, st);
  {  // q, k, v in one launch: three column blocks, each with its own weights, bias and adapter segments
    Gemm2Args g = wg_begin(c, T);
    const int tq = tiles256(D.QD), tk = tiles256(D.KVD);
    const int t0[3] = {0, tq, tq + tk}, ns[3] = {D.QD, D.KVD, D.KVD};
    bf* dst[3] = {sv->q, sv->k, sv->v};
    for (int t = 0; t < 3; ++t) {
      const int t1 = t0[t] + (t == 0 ? tq : tk);
      wg_proj(c, g, L, t, sv->h, sv, t0[t], t1);
      g.out[t] = Gemm2Out{t0[t], ns[t], dst[t], ns[t], nullptr, nullptr, 0};
    }
    g.nout = 3;
    g.tiles_n = tq + 2 * tk;
    RUN(gemm2_launch(g, st));
  }
  ft_rope(sv->q, T, S, D.nq, D.d, c->dw.inv_freq, false, c->dw.err_flag, st);
  ft_rope(sv->k, T, S, D.nkv, D.d, c->dw.inv_freq, false, c->dw.err_flag, st);
  {
    TransposeJobs tj{};
    tj.in[0] = sv->v, tj.out[0] = w.vT, tj.C[0] = D.KVD, tj.n = 1;
    ft_transpose_heads(tj, B_f, S, st);
  }
  RUN(ft_attn_fwd(sv->q, sv->k, w.vT, sv->o, sv->lse, B_f, S, D.nq, D.nkv, D.d, st));
  {  // x1 = X + o Wo^T
    proj_us_group(c, 3, 3, sv->o, T, sv, st);
    Gemm2Args g = wg_begin(c, T);
    wg_proj(c, g, L, 3, sv->o, sv, 0, tiles256(D.H));
    wg_out_f32(g, sv->x1, X, D.H);
    RUN(gemm2_launch(g, st));
  }
  ft_rmsnorm_fwd(sv->x1, L.g2, sv->h2, sv->rho2, T, D.H, m.rms_eps, c->dw.err_flag, st);
  proj_us_group(c, 4, 5, sv->h2, T, sv, st);
  {  // gate and up as one launch of interleaved pairs; the epilogue writes a, u and m = silu(a) * u
    Gemm2Args g = wg_begin(c, T);
    const int tp = (D.F + 127) / 128;  // a tile holds 128 gate + 128 up columns
    wg_seg(g, sv->h2, D.H, D.H, L.w16[4], D.F, 0, tp, L.w16[5], 1);
    const int r = c->lora.rank;
    if (adapted(c, 4)) wg_seg(g, sv->us[4], r, r, w.Bt[4], D.F, 0, tp, nullptr, 1);
    if (adapted(c, 5)) wg_seg(g, sv->us[5], r, r, nullptr, D.F, 0, tp, w.Bt[5], 1);
    g.epi = GEMM2_EPI_GATEUP;
    g.nout = 1;
    g.tiles_n = tp;
    g.out[0] = Gemm2Out{0, D.F, sv->a, D.F, nullptr, nullptr, 0};
    g.o1 = sv->u;
    g.o0 = sv->m;
    g.lde = D.F;
    RUN(gemm2_launch(g, st));
  }
  {  // Y = x1 + m Wd^T
    proj_us_group(c, 6, 6, sv->m, T, sv, st);
    Gemm2Args g = wg_begin(c, T);
    wg_proj(c, g, L, 6, sv->m, sv, 0, tiles256(D.H));
    wg_out_f32(g, Y, sv->x1, D.H);
    RUN(gemm2_launch(g, st));
  }
  if (hipGetLastError() != hipSuccess) {
    release_saved(c, sv, st, true);
    return fail(HARLI_ERR_HIP, "lora_fwd: a kernel launch failed");
  }
  s = window_release(c, layer, false, st);
  if (s != HARLI_OK) {
    release_saved(c, sv, st, true);
    return s;
  }
  *saved = sv;
  return HARLI_OK;
}

extern "C" harli_status harli_lora_bwd(harli_ctx* c, int32_t layer, const float* dY, float* dX, harli_saved* sv,
                                       float* const* dA, float* const* dB, void* hip_stream) {
  if (!sv) return fail(HARLI_ERR_INVALID, "lora_bwd: null saved record");
  harli_status s = check_call(c, layer, sv->Bf, sv->S, "lora_bwd");
  if (s != HARLI_OK) return s;
  if (!dY || !dX || !dA || !dB) return fail(HARLI_ERR_INVALID, "lora_bwd: null argument");
  if (sv->layer != layer) return fail(HARLI_ERR_INVALID, "lora_bwd: saved record belongs to layer %d", sv->layer);
  for (int t = 0; t < kTargets; ++t)
    if (adapted(c, t) && (!dA[t] || !dB[t])) return fail(HARLI_ERR_INVALID, "lora_bwd: null gradient buffer for target %d", t);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int B_f = sv->Bf, S = sv->S;
  const Dims D = dims(c, B_f, S);
  const LayerDev& L = c->layers[layer];
  s = ensure_ws(c, B_f, S);
  if (s != HARLI_OK) return s;
  FtWs& w = state(c)->ws;
  s = window_acquire(c, layer, true, st);
  if (s != HARLI_OK) return s;
  const int T = D.T;

#define RUNB(x)                         \
  do {                                  \
    harli_status r_ = (x);              \
    if (r_ != HARLI_OK) return r_;      \
  } while (0)

  // ---- FFN ----
  convert_adapters(c, L, false, st);
  // every gradient below carries the factor sigma
  ft_scale_to_e(dY, w.dyb, (long long)T * D.H, w.scale, w.scale_parity++, 8 - c->lora.grad_headroom_log2, st);
  const int r = c->lora.rank;
  {  // dm = dy Wd (+ gs A_d^T) -> da, du
    Gemm2Args g = wg_begin(c, T);
    const int tf = tiles256(D.F);
    wg_seg(g, w.dyb, D.H, D.H, L.wt[6], D.F, 0, tf);
    if (adapted(c, 6)) {
      RUNB(proj_grads(c, L, 6, 0, w.dyb, sv->m, T, sv, dA, dB, st));
      wg_seg(g, w.gs[0], r, r, w.An[6], D.F, 0, tf);
    }
    // the epilogue turns dm straight into da and du (SwiGLU backward); dm itself is never stored
    g.epi = GEMM2_EPI_SWIGLU_BWD;
    g.e0 = sv->a; g.e1 = sv->u; g.o0 = w.da; g.o1 = w.du; g.lde = D.F;
    g.nout = 1;
    g.tiles_n = tf;
    g.out[0] = Gemm2Out{0, D.F, nullptr, 0, nullptr, nullptr, 0};
    RUNB(gemm2_launch(g, st));
  }
  {  // dh2 = da Wg + du Wu
    Gemm2Args g = wg_begin(c, T);
    const int th = tiles256(D.H);
    wg_seg(g, w.da, D.F, D.F, L.wt[4], D.H, 0, th);
    wg_seg(g, w.du, D.F, D.F, L.wt[5], D.H, 0, th);
    {
      int ts[2], slots[2], n = 0;
      const bf* dys[2];
      for (int t = 4; t <= 5; ++t)
        if (adapted(c, t)) ts[n] = t, slots[n] = t - 4, dys[n] = t == 4 ? w.da : w.du, ++n;
      if (n) RUNB(proj_grads_group(c, n, ts, slots, dys, sv->h2, T, sv, dA, dB, st));
      for (int i = 0; i < n; ++i) wg_seg(g, w.gs[slots[i]], r, r, w.An[ts[i]], D.H, 0, th);  // dh2 += gs_t A_t^T as one more K segment
    }
    wg_out_f32(g, w.dh2, nullptr, D.H);
    RUNB(gemm2_launch(g, st));
  }
  ft_rmsnorm_bwd(w.dh2, sv->x1, sv->rho2, L.g2, dY, w.dx1, w.dx1b, T, D.H, w.scale, nullptr, c->dw.err_flag, st);
  // ---- attention output projection ----
  {  // do = dx1 Wo
    Gemm2Args g = wg_begin(c, T);
    const int tq = tiles256(D.QD);
    wg_seg(g, w.dx1b, D.H, D.H, L.wt[3], D.QD, 0, tq);
    if (adapted(c, 3)) {
      RUNB(proj_grads(c, L, 3, 0, w.dx1b, sv->o, T, sv, dA, dB, st));
      wg_seg(g, w.gs[0], r, r, w.An[3], D.QD, 0, tq);
    }
    wg_out_16(g, w.dob, D.QD);
    RUNB(gemm2_launch(g, st));
  }
  // ---- attention ----
  {
    TransposeJobs tj{};
    tj.in[0] = w.dob, tj.out[0] = w.doT, tj.C[0] = D.QD;
    tj.in[1] = sv->q, tj.out[1] = w.qT, tj.C[1] = D.QD;
    tj.in[2] = sv->k, tj.out[2] = w.kT, tj.C[2] = D.KVD;
    tj.n = 3;
    ft_transpose_heads(tj, B_f, S, st);
  }
  RUNB(ft_attn_bwd(sv->q, sv->k, sv->v, sv->o, w.qT, w.kT, w.dob, w.doT, sv->lse, w.delta, w.dq, w.dkq, w.dvq, B_f, S, D.nq,
                   D.nkv, D.d, c->dw.err_flag, st));
  const bf *dk = w.dkq, *dv = w.dvq;
  if (D.G > 1) {
    ft_sum_groups(w.dkq, w.dk, T, D.nkv, D.G, D.d, c->dw.err_flag, st);
    ft_sum_groups(w.dvq, w.dv, T, D.nkv, D.G, D.d, c->dw.err_flag, st);
    dk = w.dk;
    dv = w.dv;
  }
  ft_rope(w.dq, T, S, D.nq, D.d, c->dw.inv_freq, true, c->dw.err_flag, st);
  ft_rope(const_cast<bf*>(dk), T, S, D.nkv, D.d, c->dw.inv_freq, true, c->dw.err_flag, st);
  // ---- q, k, v projections ----
  {  // dh = dq Wq + dk Wk + dv Wv
    Gemm2Args g = wg_begin(c, T);
    const int th = tiles256(D.H);
    wg_seg(g, w.dq, D.QD, D.QD, L.wt[0], D.H, 0, th);
    wg_seg(g, dk, D.KVD, D.KVD, L.wt[1], D.H, 0, th);
    wg_seg(g, dv, D.KVD, D.KVD, L.wt[2], D.H, 0, th);
    const bf* all[3] = {w.dq, dk, dv};
    {
      int ts[3], slots[3], n = 0;
      const bf* dys[3];
      for (int t = 0; t < 3; ++t)
        if (adapted(c, t)) ts[n] = t, slots[n] = t, dys[n] = all[t], ++n;
      if (n) RUNB(proj_grads_group(c, n, ts, slots, dys, sv->h, T, sv, dA, dB, st));
      for (int i = 0; i < n; ++i) wg_seg(g, w.gs[slots[i]], r, r, w.An[ts[i]], D.H, 0, th);  // dh += gs_t A_t^T as one more K segment
    }
    wg_out_f32(g, w.dh, nullptr, D.H);
    RUNB(gemm2_launch(g, st));
  }
  ft_rmsnorm_bwd(w.dh, sv->X, sv->rho1, L.g1, w.dx1, dX, nullptr, T, D.H, nullptr, w.scale + 1, c->dw.err_flag, st);
  HARLI_HIP(hipGetLastError());
  s = window_release(c, layer, true, st);
  release_saved(c, sv, st, true);
  return s;
}

extern "C" harli_status harli_saved_release(harli_ctx* c, harli_saved* saved, void* hip_stream) {
  if (!c || !saved) return fail(HARLI_ERR_INVALID, "saved_release: null argument");
  release_saved(c, saved, static_cast<hipStream_t>(hip_stream), true);
  return HARLI_OK;
}
