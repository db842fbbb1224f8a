// Window over the finetune task's frozen weights (Harli Sec. 4.3; Sec. 4.4 for the shrink under memory pressure).
#include "window.h"
#include "gemm2.h"

#include <vector>

#include "ctx.h"
#include "window_plan.h"

using namespace harli;

namespace {

struct FtWindow {
  WindowPlan plan;
  size_t item_bytes = 0;
  size_t off[kTargets] = {}, nb[kTargets] = {};  // offset of a matrix inside an item on the host, and its bytes
  char* host = nullptr;  // pinned, [2L][item_bytes] in item order
  // One pool allocation per matrix, not per slot: every matrix is smaller than a chunk, so the pool packs them into
  // tensor chunks block by block (a slot of 3.25 chunks taken as one tensor occupied four).
  struct Slot {
    harli_alloc alloc[kTargets];
    char* ptr[kTargets];
  };
  std::vector<Slot> slot;
  std::vector<hipEvent_t> ready, used;
  std::vector<char> used_valid;
  hipStream_t copy = nullptr;
  int last_item = -1;
  long long h2d_bytes = 0, hits = 0, misses = 0, refills = 0;
};

FtWindow* win(harli_ctx* c) { return static_cast<FtWindow*>(c->window); }

harli_status load(FtWindow* w, int item, int s) {
  if (w->used_valid[s]) HARLI_HIP(hipStreamWaitEvent(w->copy, w->used[s], 0));
  for (int t = 0; t < kTargets; ++t)
    HARLI_HIP(hipMemcpyAsync(w->slot[s].ptr[t], w->host + (size_t)item * w->item_bytes + w->off[t], w->nb[t], hipMemcpyHostToDevice, w->copy));
  HARLI_HIP(hipEventRecord(w->ready[s], w->copy));
  w->plan.slot_item[s] = item;
  w->h2d_bytes += (long long)w->item_bytes;
  return HARLI_OK;
}

harli_status add_slot(harli_ctx* c, FtWindow* w) {
  FtWindow::Slot sl{};
  for (int t = 0; t < kTargets; ++t) {
    harli_status s = harli_pool_alloc(c->pool, HARLI_CLS_TENSOR, w->nb[t], &sl.alloc[t]);
    if (s != HARLI_OK) {
      for (int u = 0; u < t; ++u) (void)harli_pool_free(c->pool, &sl.alloc[u], nullptr);
      return s;
    }
    sl.ptr[t] = static_cast<char*>(sl.alloc[t].ptr);
  }
  hipEvent_t r = nullptr, u = nullptr;
  if (hipEventCreateWithFlags(&r, hipEventDisableTiming) != hipSuccess || hipEventCreateWithFlags(&u, hipEventDisableTiming) != hipSuccess) {
    if (r) (void)hipEventDestroy(r);
    for (int t = 0; t < kTargets; ++t) (void)harli_pool_free(c->pool, &sl.alloc[t], nullptr);
    return fail(HARLI_ERR_HIP, "ft_window: cannot create an event");
  }
  w->slot.push_back(sl);
  w->ready.push_back(r);
  w->used.push_back(u);
  w->used_valid.push_back(0);
  w->plan.slot_item.push_back(-1);
  w->plan.n = (int)w->slot.size();
  return HARLI_OK;
}

void drop_slot(harli_ctx* c, FtWindow* w) {  // the last one; the caller has synchronised
  for (int t = 0; t < kTargets; ++t) (void)harli_pool_free(c->pool, &w->slot.back().alloc[t], nullptr);
  (void)hipEventDestroy(w->ready.back());
  (void)hipEventDestroy(w->used.back());
  w->slot.pop_back();
  w->ready.pop_back();
  w->used.pop_back();
  w->used_valid.pop_back();
  w->plan.slot_item.pop_back();
  w->plan.n = (int)w->slot.size();
}

harli_status drain(FtWindow* w) {
  HARLI_HIP(hipStreamSynchronize(w->copy));
  for (size_t s = 0; s < w->used.size(); ++s)
    if (w->used_valid[s]) HARLI_HIP(hipEventSynchronize(w->used[s]));
  return HARLI_OK;
}

// fills empty slots: first with the items the plan wants on the device from here on (in order of use), then, if slots
// are still empty, with the nearest absent items after the last one used
harli_status fill_empty(FtWindow* w) {
  const int base = w->last_item < 0 ? w->plan.items() - 1 : w->last_item;
  const std::vector<int> want = w->plan.wanted_items((base + 1) % w->plan.items(), w->plan.n);
  size_t k = 0;
  for (int s = 0; s < w->plan.n; ++s) {
    if (w->plan.slot_item[s] >= 0) continue;
    int cand = -1;
    while (k < want.size() && cand < 0) {
      if (w->plan.find(want[k]) < 0) cand = want[k];
      ++k;
    }
    for (int d = 1; d < w->plan.items() + 1 && cand < 0; ++d) {
      const int it = (base + d) % w->plan.items();
      if (w->plan.find(it) < 0) cand = it;
    }
    if (cand < 0) break;
    harli_status r = load(w, cand, s);
    if (r != HARLI_OK) return r;
  }
  return HARLI_OK;
}

}  // namespace

namespace harli {

harli_status window_acquire(harli_ctx* c, int layer, bool backward, hipStream_t st) {
  FtWindow* w = win(c);
  if (!w) return HARLI_OK;
  const int item = WindowPlan::item_of(layer, backward, w->plan.L);
  int s = w->plan.find(item);
  if (s < 0) {
    s = w->plan.victim(item);
    harli_status r = load(w, item, s);
    if (r != HARLI_OK) return r;
    w->misses += 1;
  } else {
    w->hits += 1;
  }
  HARLI_HIP(hipStreamWaitEvent(st, w->ready[s], 0));
  LayerDev& L = c->layers[layer];
  for (int t = 0; t < kTargets; ++t) (backward ? L.wt[t] : L.w16[t]) = w->slot[s].ptr[t];
  return HARLI_OK;
}

harli_status window_release(harli_ctx* c, int layer, bool backward, hipStream_t st) {
  FtWindow* w = win(c);
  if (!w) return HARLI_OK;
  const int item = WindowPlan::item_of(layer, backward, w->plan.L);
  const int s = w->plan.find(item);
  if (s < 0) return fail(HARLI_ERR_STATE, "ft_window: release of layer %d without acquire", layer);
  HARLI_HIP(hipEventRecord(w->used[s], st));
  w->used_valid[s] = 1;
  w->last_item = item;
  LayerDev& L = c->layers[layer];
  for (int t = 0; t < kTargets; ++t) (backward ? L.wt[t] : L.w16[t]) = nullptr;
  const int nxt = w->plan.refill_after(item);
  if (nxt >= 0) {
    w->refills += 1;
    return load(w, nxt, s);
  }
  return HARLI_OK;
}

// the layers' weight tables point into slots (or nowhere) while a window is in place: nothing of theirs to free
void detach_layers(harli_ctx* c) {
  for (LayerDev& Ld : c->layers)
    for (int t = 0; t < kTargets; ++t) Ld.w16[t] = Ld.wt[t] = nullptr;
}

void free_window_state(harli_ctx* c) {
  FtWindow* w = win(c);
  if (!w) return;
  // only wait when the runtime still answers (a context destroyed while the process is going down must not block)
  const hipError_t q = w->copy ? hipStreamQuery(w->copy) : hipSuccess;
  if (q == hipSuccess || q == hipErrorNotReady) (void)drain(w);
  while (!w->slot.empty()) drop_slot(c, w);
  if (w->host) (void)hipHostFree(w->host);
  if (w->copy) (void)hipStreamDestroy(w->copy);
  delete w;
  c->window = nullptr;
}

}  // namespace harli

extern "C" harli_status harli_ft_window_enable(harli_ctx* c, int32_t n_slots) {
  if (!c || n_slots < 1) return fail(HARLI_ERR_INVALID, "ft_window_enable: null context or n_slots < 1");
  if (!c->lora_attached) return fail(HARLI_ERR_STATE, "ft_window_enable: call harli_lora_attach first");
  if (c->window) return fail(HARLI_ERR_STATE, "ft_window_enable: a window is already in place");
  const int L = c->cfg.n_layers;
  FtWindow* w = new FtWindow;
  w->plan.init(L, 0);
  size_t o = 0;
  for (int t = 0; t < kTargets; ++t) {
    int out, in;
    proj_shape(c->cfg, t, &out, &in);
    w->off[t] = o;
    w->nb[t] = ft_weight_copy_bytes(out, in);
    o += (w->nb[t] + 255) / 256 * 256;
  }
  w->item_bytes = o;
  c->window = w;
  auto bail = [&](harli_status s) {  // nothing has been moved when this is used
    free_window_state(c);
    return s;
  };
  if (hipStreamCreateWithFlags(&w->copy, hipStreamNonBlocking) != hipSuccess) return bail(fail(HARLI_ERR_HIP, "ft_window_enable: cannot create the copy stream"));
  const int want = n_slots < 2 * L ? n_slots : 2 * L;
  for (int s = 0; s < want; ++s) {
    harli_status r = add_slot(c, w);
    if (r != HARLI_OK) return bail(r);  // the pool cannot hold that many slots: nothing has been moved yet
  }
  if (hipHostMalloc(reinterpret_cast<void**>(&w->host), (size_t)2 * L * w->item_bytes, hipHostMallocDefault) != hipSuccess)
    return bail(fail(HARLI_ERR_OOM, "ft_window_enable: cannot pin %zu bytes of host memory", (size_t)2 * L * w->item_bytes));
  if (hipDeviceSynchronize() != hipSuccess) return bail(fail(HARLI_ERR_HIP, "ft_window_enable: device error"));
  // move the finetune-private copies to the host: forward copies are items 0..L-1, transposed copies 2L-1..L
  for (int l = 0; l < L; ++l) {
    LayerDev& Ld = c->layers[l];
    for (int t = 0; t < kTargets; ++t) {
      int out, in;
      proj_shape(c->cfg, t, &out, &in);
      const size_t nb = ft_weight_copy_bytes(out, in);
      if (hipMemcpy(w->host + (size_t)l * w->item_bytes + w->off[t], Ld.w16[t], nb, hipMemcpyDeviceToHost) != hipSuccess ||
          hipMemcpy(w->host + (size_t)(2 * L - 1 - l) * w->item_bytes + w->off[t], Ld.wt[t], nb, hipMemcpyDeviceToHost) != hipSuccess)
        return bail(fail(HARLI_ERR_HIP, "ft_window_enable: copy to the host failed"));
    }
  }
  for (int l = 0; l < L; ++l)
    for (int t = 0; t < kTargets; ++t) {
      LayerDev& Ld = c->layers[l];
      lib_free(c, Ld.w16[t]);
      lib_free(c, Ld.wt[t]);
      Ld.w16[t] = Ld.wt[t] = nullptr;
    }
  return fill_empty(w);
}

extern "C" harli_status harli_ft_window_disable(harli_ctx* c) {
  if (!c) return fail(HARLI_ERR_INVALID, "ft_window_disable: null context");
  FtWindow* w = win(c);
  if (!w) return fail(HARLI_ERR_STATE, "ft_window_disable: no window in place");
  harli_status r = drain(w);
  if (r != HARLI_OK) return r;
  detach_layers(c);
  const int L = c->cfg.n_layers;
  for (int l = 0; l < L; ++l) {
    LayerDev& Ld = c->layers[l];
    for (int t = 0; t < kTargets; ++t) {
      int out, in;
      proj_shape(c->cfg, t, &out, &in);
      const size_t nb = ft_weight_copy_bytes(out, in);
      harli_status am = lib_alloc(c, &Ld.w16[t], nb);
      if (am == HARLI_OK) am = lib_alloc(c, &Ld.wt[t], nb);
      if (am != HARLI_OK) return am;
      HARLI_HIP(hipMemcpy(Ld.w16[t], w->host + (size_t)l * w->item_bytes + w->off[t], nb, hipMemcpyHostToDevice));
      HARLI_HIP(hipMemcpy(Ld.wt[t], w->host + (size_t)(2 * L - 1 - l) * w->item_bytes + w->off[t], nb, hipMemcpyHostToDevice));
    }
  }
  free_window_state(c);
  return HARLI_OK;
}

extern "C" harli_status harli_ft_window_resize(harli_ctx* c, int32_t n_slots) {
  if (!c || n_slots < 1) return fail(HARLI_ERR_INVALID, "ft_window_resize: null context or n_slots < 1");
  FtWindow* w = win(c);
  if (!w) return fail(HARLI_ERR_STATE, "ft_window_resize: no window in place");
  const int want = n_slots < w->plan.items() ? n_slots : w->plan.items();
  if (want == w->plan.n) return HARLI_OK;
  harli_status r = drain(w);
  if (r != HARLI_OK) return r;
  if (want < w->plan.n) {
    // drop empty slots first, then items the smaller window does not want (see wanted_items), then wanted ones; within
    // a class the item that comes latest after the last use goes first
    const int base = w->last_item < 0 ? w->plan.items() - 1 : w->last_item;
    const int N = w->plan.items();
    std::vector<char> wanted(N, 0);
    for (int it : w->plan.wanted_items((base + 1) % N, want)) wanted[it] = 1;
    auto rank = [&](int s) {
      const int it = w->plan.slot_item[s];
      if (it < 0) return 3 * N;
      const int d = w->plan.ahead(base, it);
      const int far = d == 0 ? N : d;  // the item just used is needed a whole cycle from now
      return wanted[it] ? far : N + far;
    };
    while (w->plan.n > want) {
      int far = -1, fs = -1;
      for (int s = 0; s < w->plan.n; ++s)
        if (rank(s) > far) far = rank(s), fs = s;
      // swap slot fs with the last slot, then drop the last
      const int last = w->plan.n - 1;
      std::swap(w->slot[fs], w->slot[last]);
      std::swap(w->ready[fs], w->ready[last]);
      std::swap(w->used[fs], w->used[last]);
      std::swap(w->used_valid[fs], w->used_valid[last]);
      std::swap(w->plan.slot_item[fs], w->plan.slot_item[last]);
      drop_slot(c, w);
    }
    return HARLI_OK;
  }
  while (w->plan.n < want) {
    r = add_slot(c, w);
    if (r != HARLI_OK) return r;  // the window keeps the slots it got
  }
  return fill_empty(w);
}

extern "C" harli_status harli_ft_window_ready(harli_ctx* c, int32_t layer, int32_t backward, int32_t* ready) {
  if (!c || !ready || layer < 0 || layer >= c->cfg.n_layers) return fail(HARLI_ERR_INVALID, "ft_window_ready: bad argument");
  FtWindow* w = win(c);
  if (!w) {
    *ready = 1;
    return HARLI_OK;
  }
  const int s = w->plan.find(WindowPlan::item_of(layer, backward != 0, w->plan.L));
  *ready = s >= 0 && hipEventQuery(w->ready[s]) == hipSuccess;
  return HARLI_OK;
}

extern "C" harli_status harli_ft_window_stats(harli_ctx* c, harli_window_stats* out) {
  if (!c || !out) return fail(HARLI_ERR_INVALID, "ft_window_stats: null argument");
  FtWindow* w = win(c);
  *out = harli_window_stats{};
  if (!w) return HARLI_OK;
  out->slots = w->plan.n;
  out->slot_bytes = w->item_bytes;
  out->host_bytes = (size_t)w->plan.items() * w->item_bytes;
  out->h2d_bytes = w->h2d_bytes;
  out->hits = w->hits;
  out->misses = w->misses;
  out->refills = w->refills;
  return HARLI_OK;
}

extern "C" harli_status harli_dbg_window_plan(int32_t n_layers, int32_t n_slots, const int32_t* items, int32_t n_access,
                                              int32_t* slot, int32_t* miss, int32_t* refill) {
  if (n_layers < 1 || n_slots < 1 || !items || n_access < 0 || !slot || !miss || !refill)
    return fail(HARLI_ERR_INVALID, "dbg_window_plan: bad argument");
  WindowPlan p;
  p.init(n_layers, n_slots < 2 * n_layers ? n_slots : 2 * n_layers);
  {
    const std::vector<int> start = p.wanted_items(0, p.n);  // what enable() puts on the device
    for (int s = 0; s < p.n; ++s) p.slot_item[s] = start[s];
  }
  for (int a = 0; a < n_access; ++a) {
    const int it = items[a];
    if (it < 0 || it >= p.items()) return fail(HARLI_ERR_INVALID, "dbg_window_plan: item %d out of range", it);
    int s = p.find(it);
    miss[a] = -1;
    if (s < 0) {
      s = p.victim(it);
      p.slot_item[s] = it;
      miss[a] = it;
    }
    slot[a] = s;
    refill[a] = p.refill_after(it);
    if (refill[a] >= 0) p.slot_item[s] = refill[a];
  }
  return HARLI_OK;
}

extern "C" harli_status harli_ft_window_advise(int32_t slots, int32_t max_slots, int64_t slot_chunks, int64_t free_chunks,
                                               int64_t need_chunks, int32_t pressed, int32_t* calm, int32_t* target) {
  if (slots < 1 || max_slots < slots || slot_chunks < 1 || free_chunks < 0 || need_chunks < 0 || !calm || *calm < 0 || !target)
    return fail(HARLI_ERR_INVALID, "ft_window_advise: bad argument");
  const WindowAdvice a = advise_slots(slots, max_slots, slot_chunks, free_chunks, need_chunks, pressed != 0, *calm);
  *target = a.target;
  *calm = a.calm;
  return HARLI_OK;
}
