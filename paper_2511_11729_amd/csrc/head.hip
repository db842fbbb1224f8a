// Output layer of the finetune task with next-token cross entropy (Harli Sec. 2.1: the model is an embedding, a
// stack of transformer layers and an output layer; the frozen output layer only passes the gradient down).
//   h = RMSNorm(x; g_final), logits = h W_lm^T, loss = mean NLL over counted positions, dx = dloss/dx.
// Logits exist only as a row chunk in the workspace: per chunk one MFMA GEMM makes them (fp32), one kernel turns a
// row into (softmax - onehot) in half precision and adds the row's loss, and a second GEMM multiplies by W_lm.
// The 1 / count of the mean is applied at the very end (RMSNorm backward), so the half-precision gradient of the
// logits stays in [-1, 1].
#include <algorithm>

#include "ctx.h"
#include "ft_elem.h"
#include "ft_kernels.h"
#include "gemm_timer.h"
#include "gemm2.h"

namespace harli {
namespace {

struct HeadWs {
  char* base = nullptr;
  size_t bytes = 0;
  bf *w16 = nullptr, *wT = nullptr;  // the output layer as the weight GEMM's blocked operands [V rows, H] and [H rows, V] (made once)
  bf *h = nullptr, *dlog = nullptr;
  float *rho = nullptr, *logits = nullptr, *dh = nullptr, *acc = nullptr;  // acc: [0] loss sum, [1] count, [2] 1/count
  float* rowloss = nullptr;  // [T] loss of a counted row, -1 for a row that is not counted
  int T = 0, TC = 0, Vp = 0;
  bool weights_ready = false;
  bool in_pool = false;      // base is `alloc` (a TENSOR allocation of the unified pool) rather than a library allocation
  harli_alloc alloc{};
  size_t weight_bytes = 0;
};

inline size_t al(size_t n) { return (n + 255) & ~size_t(255); }

// one workgroup per row: max, log-sum-exp, loss, and dlog = softmax - onehot (zero row when the position is not counted)
__global__ void __launch_bounds__(256) k_ce_row(const float* __restrict__ logits, const int* __restrict__ targets, bf* __restrict__ dlog,
                                                int V, int Vp, float* rowloss, int* err_flag) {
  __shared__ float red[4];
  __shared__ float bc;
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = logits + (size_t)row * Vp;
  bf* d = dlog + (size_t)row * Vp;
  int tg = targets[row];
  if (tg >= V) {
    if (tid == 0) atomicOr(err_flag, 2);
    tg = -1;
  }
  if (tg < 0) {
    for (int j = tid; j < Vp; j += 256) d[j] = 0;
    if (tid == 0) rowloss[row] = -1.f;
    return;
  }
  float mx = -INFINITY;
  for (int j = tid; j < V; j += 256) mx = fmaxf(mx, z[j]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = tid; j < V; j += 256) sum += expf(z[j] - mx);
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    const float tot = red[0] + red[1] + red[2] + red[3];
    bc = 1.f / tot;
    rowloss[row] = fmaxf(logf(tot) + mx - z[tg], 0.f);  // a row's loss is >= 0; rounding may leave -0
  }
  __syncthreads();
  const float inv = bc;
  for (int j = tid; j < Vp; j += 256) {
    float p = j < V ? expf(z[j] - mx) * inv : 0.f;
    if (j == tg) p -= 1.f;
    d[j] = F2E(p);
  }
}

// Sum of the rows' losses in a fixed order (thread t takes rows t, t + 256, ..., then a tree over the threads), so
// that the loss is the same number in every run; atomics would add the rows in the order they happen to finish.
__global__ void __launch_bounds__(256) k_head_finish(const float* rowloss, int T, float* acc, float* loss) {
  __shared__ float sl[256];
  __shared__ int sn[256];
  const int tid = threadIdx.x;
  float l = 0.f;
  int n = 0;
  for (int r = tid; r < T; r += 256) {
    const float v = rowloss[r];
    if (v >= 0.f) l += v, ++n;
  }
  sl[tid] = l;
  sn[tid] = n;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) sl[tid] += sl[tid + o], sn[tid] += sn[tid + o];
    __syncthreads();
  }
  if (tid == 0) {
    const float cnt = fmaxf((float)sn[0], 1.f);
    acc[0] = sl[0];
    acc[1] = (float)sn[0];
    acc[2] = 1.f / cnt;
    *loss = sl[0] / cnt;
  }
}

HeadWs* ws_of(harli_ctx* c) { return static_cast<HeadWs*>(c->head_ws); }

harli_status head_free_ws(harli_ctx* c) {
  HeadWs* w = ws_of(c);
  if (!w || !w->base) return HARLI_OK;
  HARLI_HIP(hipDeviceSynchronize());
  if (w->in_pool) {
    harli_status r = harli_pool_free(c->pool, &w->alloc, nullptr);
    if (r != HARLI_OK) return r;
  } else {
    HARLI_HIP(hipFree(w->base));
  }
  w->base = nullptr;
  w->bytes = 0;
  w->in_pool = false;
  return HARLI_OK;
}

}  // namespace

// Made once when the adapters are attached (the context has an output layer): the blocked copies of the output layer
// and the workspace for max_ft_tokens rows -- from the unified pool when the adapters were attached with
// workspace_in_pool, else a library allocation -- so that harli_head_fwd_bwd itself allocates nothing.
harli_status head_prepare(harli_ctx* c) {
  if (!c->w_lm || !c->g_final || c->cfg.vocab < 1) return HARLI_OK;
  if (!c->head_ws) c->head_ws = new HeadWs;
  HeadWs& w = *ws_of(c);
  const int V = c->cfg.vocab, H = c->cfg.hidden, T = c->cfg.max_ft_tokens;
  const int Vp = (V + 7) & ~7;
  if (!w.weights_ready) {
    harli_status am = lib_alloc(c, reinterpret_cast<void**>(&w.w16), blocked_elems(V, H) * 2);
    if (am == HARLI_OK) am = lib_alloc(c, reinterpret_cast<void**>(&w.wT), blocked_elems(H, Vp) * 2);
    if (am != HARLI_OK) {
      lib_free(c, w.w16);
      w.w16 = w.wT = nullptr;
      return am;
    }
    const int f32 = c->cfg.dtype == HARLI_F32 ? 1 : 0;
    BlockJobs jobs{};
    jobs.half = 1;
    jobs.flag = c->dw.err_flag;  // an output-layer weight beyond the element's range shows in harli_ctx_check
    jobs.j[jobs.n++] = BlockJob{c->w_lm, w.w16, V, H, 0, f32};  // operand [n = class][k = hidden]
    jobs.j[jobs.n++] = BlockJob{c->w_lm, w.wT, V, H, 1, f32};   // operand [n = hidden][k = class], zero past V
    gemm2_block_jobs(jobs, nullptr);
    HARLI_HIP(hipDeviceSynchronize());
    w.Vp = Vp;
    w.weight_bytes = (blocked_elems(V, H) + blocked_elems(H, Vp)) * 2;
    w.weights_ready = true;
  }
  // row chunk: at most 2048 rows and about 512 MiB of fp32 logits
  const int TC = (int)std::max<long long>(64, std::min<long long>(2048, ((512ll << 20) / ((long long)Vp * 4)) / 64 * 64));
  size_t off = 0;
  auto take = [&](size_t n) {
    size_t o = off;
    off += al(n);
    return o;
  };
  const size_t o_h = take((size_t)T * H * 2), o_rho = take((size_t)T * 4), o_log = take((size_t)TC * Vp * 4);
  const size_t o_dlog = take((size_t)TC * Vp * 2), o_dh = take((size_t)T * H * 4), o_acc = take(64), o_rl = take((size_t)T * 4);
  const bool want_pool = c->lora.workspace_in_pool != 0 || c->cfg.memory_in_pool != 0;
  if (off != w.bytes || want_pool != w.in_pool) {
    harli_status r = head_free_ws(c);
    if (r != HARLI_OK) return r;
    if (want_pool) {
      r = harli_pool_alloc(c->pool, HARLI_CLS_TENSOR, off, &w.alloc);
      if (r != HARLI_OK) return r;
      w.base = static_cast<char*>(w.alloc.ptr);
    } else {
      HARLI_HIP(hipMalloc(reinterpret_cast<void**>(&w.base), off));
    }
    w.in_pool = want_pool;
    w.bytes = off;
  }
  char* b = w.base;
  w.h = (bf*)(b + o_h); w.rho = (float*)(b + o_rho); w.logits = (float*)(b + o_log); w.dlog = (bf*)(b + o_dlog);
  w.dh = (float*)(b + o_dh); w.acc = (float*)(b + o_acc); w.rowloss = (float*)(b + o_rl);
  w.T = T;
  w.TC = TC;
  return HARLI_OK;
}

void head_device_bytes(const harli_ctx* c, size_t* weights, size_t* workspace, int* in_pool) {
  *weights = *workspace = 0;
  *in_pool = 0;
  if (!c->head_ws) return;
  const HeadWs* w = static_cast<const HeadWs*>(c->head_ws);
  *weights = w->weight_bytes;
  *workspace = w->bytes;
  *in_pool = w->in_pool ? 1 : 0;
}

void free_head_state(harli_ctx* c) {
  if (!c->head_ws) return;
  HeadWs* w = ws_of(c);
  (void)head_free_ws(c);
  lib_free(c, w->w16);
  lib_free(c, w->wT);
  delete w;
  c->head_ws = nullptr;
}

}  // namespace harli

extern "C" harli_status harli_head_fwd_bwd(harli_ctx* c, const float* x, const int32_t* targets, int32_t T, float* loss, float* dx,
                                           void* hip_stream) {
  using namespace harli;
  if (!c || !x || !targets || !loss || !dx) return fail(HARLI_ERR_INVALID, "head_fwd_bwd: null argument");
  if (!c->lora_attached) return fail(HARLI_ERR_STATE, "head_fwd_bwd: call harli_lora_attach first");
  if (!c->w_lm || !c->g_final || c->cfg.vocab < 1) return fail(HARLI_ERR_STATE, "head_fwd_bwd: the context has no output layer (g_final, w_lm, vocab)");
  if (T < 1 || T > c->cfg.max_ft_tokens) return fail(HARLI_ERR_INVALID, "head_fwd_bwd: %d tokens outside 1..max_ft_tokens %d", T, c->cfg.max_ft_tokens);
  if (c->cfg.hidden % 8) return fail(HARLI_ERR_INVALID, "head_fwd_bwd: hidden must be a multiple of 8");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (!c->head_ws || !ws_of(c)->base) return fail(HARLI_ERR_STATE, "head_fwd_bwd: the output layer was not prepared by harli_lora_attach");
  harli_status s = HARLI_OK;
  HeadWs& w = *ws_of(c);
  const int V = c->cfg.vocab, H = c->cfg.hidden, Vp = w.Vp;
  ft_rmsnorm_fwd(x, c->g_final, w.h, w.rho, T, H, c->cfg.rms_eps, c->dw.err_flag, st);
  for (int t0 = 0; t0 < T; t0 += w.TC) {
    const int rows = std::min(w.TC, T - t0);
    {  // logits = h W^T
      Gemm2Args g{};
      g.M = rows; g.alpha = 1.f; g.half = 1; g.overflow_flag = c->dw.err_flag;
      g.nseg = 1;
      g.seg[0] = Gemm2Seg{w.h + (size_t)t0 * H, H, H, w.w16, 0, (V + kG2TileN - 1) / kG2TileN, nullptr, 0, V};
      g.nout = 1;
      g.tiles_n = (V + kG2TileN - 1) / kG2TileN;
      g.out[0] = Gemm2Out{0, V, nullptr, 0, w.logits, nullptr, Vp};
      s = gemm2_launch(g, st);
      if (s != HARLI_OK) return s;
    }
    hipLaunchKernelGGL(k_ce_row, dim3(rows), dim3(256), 0, st, w.logits, targets + t0, w.dlog, V, Vp, w.rowloss + t0, c->dw.err_flag);
    {  // dh = dlog W   (contraction over the padded vocabulary: pad columns are zero on both sides)
      Gemm2Args g{};
      g.M = rows; g.alpha = 1.f; g.half = 1; g.overflow_flag = c->dw.err_flag;
      g.nseg = 1;
      g.seg[0] = Gemm2Seg{w.dlog, Vp, Vp, w.wT, 0, (H + kG2TileN - 1) / kG2TileN, nullptr, 0, H};
      g.nout = 1;
      g.tiles_n = (H + kG2TileN - 1) / kG2TileN;
      g.out[0] = Gemm2Out{0, H, nullptr, 0, w.dh + (size_t)t0 * H, nullptr, H};
      s = gemm2_launch(g, st);
      if (s != HARLI_OK) return s;
    }
  }
  hipLaunchKernelGGL(k_head_finish, dim3(1), dim3(256), 0, st, w.rowloss, T, w.acc, loss);
  ft_rmsnorm_bwd(w.dh, x, w.rho, c->g_final, nullptr, dx, nullptr, T, H, nullptr, w.acc + 2, c->dw.err_flag, st);
  HARLI_HIP(hipGetLastError());
  return HARLI_OK;
}
