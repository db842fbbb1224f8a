// Model context: shapes, borrowed weight pointers and the library-owned device workspace.
#include "ctx.h"

#include "decode_large.h"

#include <cmath>

using namespace harli;

namespace harli {

int event_done(void* hip_event) {
  hipError_t e = hipEventQuery(static_cast<hipEvent_t>(hip_event));
  if (e == hipSuccess) return 1;
  if (e == hipErrorNotReady) return 0;
  (void)hipGetLastError();
  return -1;
}

void event_destroy(void* hip_event) { (void)hipEventDestroy(static_cast<hipEvent_t>(hip_event)); }

harli_status lib_alloc(harli_ctx* c, void** p, size_t bytes) {
  if (bytes == 0) bytes = 16;
  if (!c->cfg.memory_in_pool) {
    HARLI_HIP(hipMalloc(p, bytes));
    return HARLI_OK;
  }
  harli_alloc a{};
  harli_status s = harli_pool_alloc(c->pool, HARLI_CLS_AUTO, bytes, &a);
  if (s != HARLI_OK) return s;
  c->pool_allocs[a.ptr] = a;
  *p = a.ptr;
  return HARLI_OK;
}
void lib_free(harli_ctx* c, void* p) {
  if (!p) return;
  auto it = c->pool_allocs.find(p);
  if (it == c->pool_allocs.end()) {
    (void)hipFree(p);
    return;
  }
  (void)harli_pool_free(c->pool, &it->second, nullptr);
  c->pool_allocs.erase(it);
}

static size_t g_tally = 0;  // bytes handed out by dev_alloc since the caller last read it (harli_ctx_create is not re-entrant)
template <typename T>
static harli_status dev_alloc(harli_ctx* c, T** p, size_t bytes, bool zero) {
  harli_status s = lib_alloc(c, reinterpret_cast<void**>(p), bytes);
  if (s != HARLI_OK) return s;
  if (zero) HARLI_HIP(hipMemset(*p, 0, bytes ? bytes : 16));
  g_tally += bytes ? bytes : 16;
  return HARLI_OK;
}

void free_finetune_state(harli_ctx* c);  // finetune.hip
void finetune_device_bytes(const harli_ctx* c, size_t* weights, size_t* workspace, int* in_pool);  // finetune.hip
void head_device_bytes(const harli_ctx* c, size_t* weights, size_t* workspace, int* in_pool);      // head.hip
void free_head_state(harli_ctx* c);      // head.hip
void free_window_state(harli_ctx* c);    // window.hip
void pool_retain(harli_pool* p);          // pool.cpp
void pool_release(harli_pool* p);
void detach_layers(harli_ctx* c);        // window.hip

}  // namespace harli

#define TRY(x)                       \
  do {                               \
    harli_status s_ = (x);           \
    if (s_ != HARLI_OK) {            \
      harli_ctx_destroy(c);          \
      return s_;                     \
    }                                \
  } while (0)

extern "C" harli_status harli_ctx_create(const harli_model_cfg* cfg, const harli_weights* w, harli_pool* pool,
                                         harli_ctx** out) {
  if (!cfg || !w || !pool || !out || !w->layers) return fail(HARLI_ERR_INVALID, "ctx_create: null argument");
  const harli_model_cfg& m = *cfg;
  if (m.n_layers < 1 || m.hidden < 1 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.head_dim < 2 || m.ffn < 1)
    return fail(HARLI_ERR_INVALID, "ctx_create: non-positive shape");
  if (m.n_q_heads % m.n_kv_heads != 0) return fail(HARLI_ERR_INVALID, "ctx_create: n_q_heads %% n_kv_heads != 0");
  if (m.head_dim % 2 != 0) return fail(HARLI_ERR_INVALID, "ctx_create: head_dim must be even (rotary pairs)");
  if (m.dtype != HARLI_BF16 && m.dtype != HARLI_F32) return fail(HARLI_ERR_INVALID, "ctx_create: unknown dtype");
  if (m.max_batch < 1 || m.max_batch > 256) return fail(HARLI_ERR_INVALID, "ctx_create: max_batch outside 1..256");
  if (m.max_seq_len < 1) return fail(HARLI_ERR_INVALID, "ctx_create: max_seq_len must be positive");
  if (m.max_ft_tokens < 0) return fail(HARLI_ERR_INVALID, "ctx_create: negative max_ft_tokens");
  const int QD = m.n_q_heads * m.head_dim;
  if (m.dtype == HARLI_BF16) {
    if (m.head_dim != 64 && m.head_dim != 128)
      return fail(HARLI_ERR_INVALID, "ctx_create: bf16 kernels support head_dim 64 or 128, got %d", m.head_dim);
    if (m.hidden % 8 || m.ffn % 8 || QD % 8)
      return fail(HARLI_ERR_INVALID, "ctx_create: bf16 kernels need hidden, ffn and n_q*head_dim to be multiples of 8");
    const int G = m.n_q_heads / m.n_kv_heads;
    if (G < 1 || G > 8 || (m.head_dim == 64 && G != 1 && G != 2 && G != 4))
      return fail(HARLI_ERR_INVALID, "ctx_create: query/KV head ratio %d is not supported at head_dim %d", G, m.head_dim);
  }
  KvGeom geom;
  harli_pool_geom(pool, &geom);
  const size_t eb = m.dtype == HARLI_BF16 ? 2 : 4;
  if (geom.n_layers != m.n_layers) return fail(HARLI_ERR_INVALID, "ctx_create: pool has %d layers, model %d", geom.n_layers, m.n_layers);
  if (geom.row_bytes != (unsigned long long)m.n_kv_heads * m.head_dim * eb)
    return fail(HARLI_ERR_INVALID, "ctx_create: pool kv_row_bytes %llu != n_kv*head_dim*elem %zu", geom.row_bytes,
                (size_t)m.n_kv_heads * m.head_dim * eb);
  if (geom.page_tokens != 16) return fail(HARLI_ERR_INVALID, "ctx_create: kernels are built for 16-token pages");
  for (int l = 0; l < m.n_layers; ++l) {
    const harli_layer_weights& lw = w->layers[l];
    if (!lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.wg || !lw.wu || !lw.wd || !lw.g1 || !lw.g2)
      return fail(HARLI_ERR_INVALID, "ctx_create: layer %d has a null weight pointer", l);
  }
  if ((w->emb || w->w_lm) && m.vocab < 1) return fail(HARLI_ERR_INVALID, "ctx_create: vocab must be positive");

  harli_ctx* c = new harli_ctx;
  c->cfg = m;
  c->pool = pool;
  pool_retain(pool);
  c->geom = geom;
  c->slab = static_cast<char*>(harli_pool_slab(pool));
  c->layers.resize(m.n_layers);
  for (int l = 0; l < m.n_layers; ++l) {
    const harli_layer_weights& lw = w->layers[l];
    LayerDev& d = c->layers[l];
    const void* ws[kTargets] = {lw.wq, lw.wk, lw.wv, lw.wo, lw.wg, lw.wu, lw.wd};
    for (int t = 0; t < kTargets; ++t) {
      d.w[t] = ws[t];
      d.wt[t] = nullptr;
      d.wp[t] = nullptr;
      d.w16[t] = nullptr;
      d.A[t] = d.B[t] = nullptr;
    }
    d.g1 = lw.g1;
    d.g2 = lw.g2;
    d.bias[0] = lw.bq;
    d.bias[1] = lw.bk;
    d.bias[2] = lw.bv;
    d.b16[0] = d.b16[1] = d.b16[2] = nullptr;
  }
  c->emb = w->emb;
  c->g_final = w->g_final;
  c->w_lm = w->w_lm;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    delete c;
    return fail(HARLI_ERR_HIP, "ctx_create: no HIP device available");
  }
  c->n_cu = prop.multiProcessorCount;

  DecodeWs& d = c->dw;
  g_tally = 0;
  d.bpad = (m.max_batch + 15) / 16 * 16;
  d.max_chunks = (m.max_seq_len + 127) / 128;  // the smallest attention chunk is 128 tokens
  const size_t bp = d.bpad;
  TRY(dev_alloc(c, &d.hx1, bp * m.hidden * 4, true));
  TRY(dev_alloc(c, &d.obuf, bp * QD * 4, true));
  TRY(dev_alloc(c, &d.hx2, bp * m.hidden * 4, true));
  TRY(dev_alloc(c, &d.mbuf, bp * m.ffn * 4, true));
  TRY(dev_alloc(c, &d.qbuf, bp * QD * 4, true));
  TRY(dev_alloc(c, &d.x1, bp * m.hidden * 4, true));
  TRY(dev_alloc(c, &d.xa, bp * m.hidden * 4, true));
  TRY(dev_alloc(c, &d.xb, bp * m.hidden * 4, true));
  TRY(dev_alloc(c, &d.ssq, bp * (2 * m.n_layers + 1) * (size_t)ssq_entries(m.hidden) * 4, true));
  TRY(dev_alloc(c, &d.rope, bp * m.head_dim * 4, true));
  if (m.vocab > 0) {
    TRY(dev_alloc(c, &d.amax_v, bp * 64 * 4, true));
    TRY(dev_alloc(c, &d.amax_i, bp * 64 * 4, true));
  }
  {
    TRY(dev_alloc(c, &d.inv_freq, (m.head_dim / 2) * sizeof(double), false));
    std::vector<double> f(m.head_dim / 2);
    for (int i = 0; i < m.head_dim / 2; ++i) f[i] = std::pow((double)m.rope_base, -2.0 * i / (double)m.head_dim);
    if (hipMemcpy(d.inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess) {
      harli_ctx_destroy(c);
      return fail(HARLI_ERR_HIP, "ctx_create: copying the rotary table failed");
    }
  }
  TRY(dev_alloc(c, &d.att_part, bp * m.n_q_heads * d.max_chunks * (m.head_dim + 2) * 4, true));
  TRY(dev_alloc(c, &d.err_flag, 16, true));
  d.part_bytes = dg_workspace_bytes(m, c->n_cu);
  if (d.part_bytes) {
    TRY(dev_alloc(c, &d.part, d.part_bytes, false));
    TRY(dg_init());
  }
  // fp32 path: scratch for attention scores, one row of max_seq_len per (sequence, query head)
  if (m.dtype == HARLI_F32) {
    TRY(dev_alloc(c, &d.scores, bp * m.n_q_heads * (size_t)m.max_seq_len * 4, true));
    TRY(dev_alloc(c, &d.fk, bp * m.n_kv_heads * m.head_dim * 4, true));
    TRY(dev_alloc(c, &d.fv, bp * m.n_kv_heads * m.head_dim * 4, true));
    TRY(dev_alloc(c, &d.fa, bp * m.ffn * 4, true));
    TRY(dev_alloc(c, &d.fu, bp * m.ffn * 4, true));
  }
  c->decode_ws_bytes = g_tally;
  g_tally = 0;
  // decode-private pre-shuffled weights (bf16 path): the inference instance keeps its own copy
  if (m.dtype == HARLI_BF16) {
    const int KVD = m.n_kv_heads * m.head_dim;
    for (int l = 0; l < m.n_layers; ++l) {
      LayerDev& ld = c->layers[l];
      TRY(dev_alloc(c, &ld.wp[0], packed_weight_elems(QD + 2 * KVD, m.hidden) * 2, false));
      TRY(pack_weight(ld.w[0], ld.wp[0], QD, m.hidden, 0, nullptr));
      TRY(pack_weight(ld.w[1], ld.wp[0], KVD, m.hidden, QD / 16, nullptr));
      TRY(pack_weight(ld.w[2], ld.wp[0], KVD, m.hidden, (QD + KVD) / 16, nullptr));
      for (int t = 3; t < kTargets; ++t) {
        int o, i;
        proj_shape(m, t, &o, &i);
        TRY(dev_alloc(c, &ld.wp[t], packed_weight_elems(o, i) * 2, false));
        TRY(pack_weight(ld.w[t], ld.wp[t], o, i, 0, nullptr));
      }
    }
    if (c->w_lm) {
      TRY(dev_alloc(c, &c->wlm_p, packed_weight_elems(m.vocab, m.hidden) * 2, false));
      TRY(pack_weight(c->w_lm, c->wlm_p, m.vocab, m.hidden, 0, nullptr));
    }
    if (hipDeviceSynchronize() != hipSuccess) {
      harli_ctx_destroy(c);
      return fail(HARLI_ERR_HIP, "ctx_create: pre-shuffling the weights failed");
    }
  }
  c->decode_weight_bytes = g_tally;
  *out = c;
  return HARLI_OK;
}

extern "C" harli_status harli_ctx_device_bytes(const harli_ctx* c, harli_device_bytes* out) {
  if (!c || !out) return fail(HARLI_ERR_INVALID, "ctx_device_bytes: null argument");
  harli_device_bytes b{};
  b.decode_weights = c->decode_weight_bytes;
  b.decode_workspace = c->decode_ws_bytes;
  int ft_pool = 0, head_pool = 0;
  finetune_device_bytes(c, &b.finetune_weights, &b.finetune_workspace, &ft_pool);
  head_device_bytes(c, &b.head_weights, &b.head_workspace, &head_pool);
  const size_t all = b.decode_weights + b.decode_workspace + b.finetune_weights + b.finetune_workspace + b.head_weights + b.head_workspace;
  b.in_pool = c->cfg.memory_in_pool ? all : (ft_pool ? b.finetune_workspace : 0) + (head_pool ? b.head_workspace : 0);
  b.outside_pool = all - b.in_pool;
  *out = b;
  return HARLI_OK;
}

extern "C" void harli_ctx_destroy(harli_ctx* c) {
  if (!c) return;
  DecodeWs& d = c->dw;
  void* bufs[] = {d.hx1, d.obuf, d.hx2, d.mbuf, d.qbuf, d.x1, d.xa, d.xb, d.ssq, d.rope, d.att_part, d.amax_v, d.amax_i, d.err_flag, d.part, d.scores, d.inv_freq, d.fk, d.fv, d.fa, d.fu};
  (void)hipDeviceSynchronize();  // steps in flight may still read what goes back to the pool here
  for (void* p : bufs) lib_free(c, p);
  for (LayerDev& ld : c->layers)
    for (int t = 0; t < kTargets; ++t) lib_free(c, ld.wp[t]);
  lib_free(c, c->wlm_p);
  if (c->window) detach_layers(c);  // the weight tables point into window slots
  free_window_state(c);
  free_finetune_state(c);
  free_head_state(c);
  pool_release(c->pool);
  delete c;
}

extern "C" harli_status harli_ctx_check(harli_ctx* c, void* hip_stream) {
  if (!c) return fail(HARLI_ERR_INVALID, "ctx_check: null context");
  int flag = 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  HARLI_HIP(hipMemcpyAsync(&flag, c->dw.err_flag, sizeof(int), hipMemcpyDeviceToHost, st));
  HARLI_HIP(hipStreamSynchronize(st));
  if (flag) {
    HARLI_HIP(hipMemsetAsync(c->dw.err_flag, 0, sizeof(int), st));
    HARLI_HIP(hipStreamSynchronize(st));
    return fail(HARLI_ERR_INVALID, "a kernel saw %s%s%s%s", (flag & 1) ? "a page id outside the pool; " : "",
                (flag & 2) ? "a token or class id outside the vocabulary; " : "",
                (flag & 4) ? "a sequence longer than max_kv_len or its page-table row; " : "",
                (flag & 8) ? "a finetune activation beyond the range of the 16-bit compute element; " : "");
  }
  return HARLI_OK;
}
