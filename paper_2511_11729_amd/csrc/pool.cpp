// Unified memory pool (Harli Sec. 4.2 two-level chunk/block management, Sec. 4.4
// inference priority through a reserve, Sec. 4.5 small-tensor buddy pool).
//
// Pure host bookkeeping over one caller-owned device slab: the slab pointer is
// only ever used for address arithmetic.  Placement is "lowest index first"
// throughout so that page ids and byte offsets are reproducible.
#include <cstdio>
#include <cstring>
#include <map>
#include <cmath>
#include <atomic>
#include <mutex>
#include <set>
#include <string>
#include <unordered_map>
#include <vector>

#include "common.h"

namespace harli {

static thread_local std::string g_err;

harli_status fail(harli_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return s;
}

enum ChunkClass : uint8_t { C_FREE = 0, C_KV = 1, C_TENSOR = 2 };

struct Bitmap {
  std::vector<uint64_t> w;
  int n = 0, used = 0;
  void reset(int bits) {
    n = bits;
    used = 0;
    w.assign((bits + 63) / 64, 0);
  }
  bool get(int i) const { return (w[i >> 6] >> (i & 63)) & 1; }
  void set(int i) {
    w[i >> 6] |= 1ull << (i & 63);
    ++used;
  }
  void clr(int i) {
    w[i >> 6] &= ~(1ull << (i & 63));
    --used;
  }
  int first_zero() const {
    for (size_t k = 0; k < w.size(); ++k) {
      uint64_t inv = ~w[k];
      if (inv) {
        int i = int(k * 64) + __builtin_ctzll(inv);
        return i < n ? i : -1;
      }
    }
    return -1;
  }
  // lowest start of a run of `len` zero bits, or -1
  int first_zero_run(int len) const {
    int run = 0;
    for (int i = 0; i < n; ++i) {
      run = get(i) ? 0 : run + 1;
      if (run == len) return i - len + 1;
    }
    return -1;
  }
};

struct Live {
  int32_t cls;
  size_t bytes, requested;
};

struct Pending {
  void* event;
  bool own;  // the pool destroys the event once it has completed
  bool is_page;
  int32_t page;
  size_t offset;
};

}  // namespace harli

using namespace harli;

struct harli_pool {
  std::mutex mu;
  // the creator's reference plus one per context built on the pool: a context gives pool memory back when it is
  // destroyed, so the pool object has to live until the last of them is gone, whichever is destroyed first
  std::atomic<int> refs{1};
  char* slab = nullptr;
  size_t slab_bytes = 0;
  harli_pool_cfg cfg{};
  size_t page_bytes = 0, chunk_bytes = 0;
  int ppb = 0, bpc = 0, n_chunks = 0, max_order = 0;

  std::vector<uint8_t> cls;
  std::vector<Bitmap> bits;          // KV: page slots; TENSOR: blocks
  std::set<int> free_chunks;         // FREE chunks, ascending
  std::set<int> kv_partial;          // KV chunks with at least one free slot
  std::set<int> tensor_chunks;       // TENSOR chunks, ascending
  std::vector<std::set<size_t>> buddy;  // per order: free offsets
  std::unordered_map<size_t, Live> live;
  std::vector<Pending> pending;
  int64_t kv_pages_live = 0, tensor_blocks_live = 0, small_fallbacks = 0;
  size_t small_bytes_live = 0, requested_live = 0, reserved_live = 0;

  size_t chunk_base(int c) const { return cfg.small_pool_bytes + size_t(c) * chunk_bytes; }

  // ---- KV pages ------------------------------------------------------------
  harli_status alloc_page(int32_t* out) {
    int c;
    if (!kv_partial.empty()) {
      c = *kv_partial.begin();
    } else {
      if (free_chunks.empty()) return fail(HARLI_ERR_OOM, "pool: no chunk left for a KV page");
      c = *free_chunks.begin();
      free_chunks.erase(free_chunks.begin());
      cls[c] = C_KV;
      bits[c].reset(ppb);
      kv_partial.insert(c);
    }
    int slot = bits[c].first_zero();
    bits[c].set(slot);
    if (bits[c].used == ppb) kv_partial.erase(c);
    ++kv_pages_live;
    *out = c * ppb + slot;
    return HARLI_OK;
  }

  harli_status check_page(int32_t page) const {
    if (page < 0 || page >= n_chunks * ppb) return fail(HARLI_ERR_INVALID, "pool: page id %d out of range", page);
    int c = page / ppb, s = page % ppb;
    if (cls[c] != C_KV || !bits[c].get(s)) return fail(HARLI_ERR_INVALID, "pool: page %d is not allocated", page);
    return HARLI_OK;
  }

  void release_page(int32_t page) {
    int c = page / ppb, s = page % ppb;
    bits[c].clr(s);
    --kv_pages_live;
    if (bits[c].used == 0) {
      kv_partial.erase(c);
      cls[c] = C_FREE;
      free_chunks.insert(c);
    } else {
      kv_partial.insert(c);
    }
  }

  // ---- tensors -----------------------------------------------------------------
  void take_chunk_for_tensor(int c) {
    free_chunks.erase(c);
    cls[c] = C_TENSOR;
    bits[c].reset(bpc);
    tensor_chunks.insert(c);
  }

  void mark_blocks(int c, int b0, int nblk) {
    for (int i = 0; i < nblk; ++i) bits[c + (b0 + i) / bpc].set((b0 + i) % bpc);
    tensor_blocks_live += nblk;
  }

  harli_status alloc_tensor(size_t nbytes, size_t requested, harli_alloc* out) {
    size_t nb = (nbytes + cfg.block_bytes - 1) / cfg.block_bytes;
    if (nb == 0) nb = 1;
    if (nb > size_t(n_chunks) * bpc) return fail(HARLI_ERR_OOM, "pool: %zu bytes exceed the slab", nbytes);
    int nblk = int(nb), c = -1, b0 = 0;
    if (nblk <= bpc) {
      for (int tc : tensor_chunks) {
        int r = bits[tc].first_zero_run(nblk);
        if (r >= 0) {
          c = tc;
          b0 = r;
          break;
        }
      }
      if (c < 0) {
        if (int(free_chunks.size()) - 1 < cfg.kv_reserve_chunks || free_chunks.empty())
          return fail(HARLI_ERR_OOM, "pool: a new tensor chunk would eat the KV reserve (%zu free, %d reserved)",
                      free_chunks.size(), cfg.kv_reserve_chunks);
        c = *free_chunks.begin();
        take_chunk_for_tensor(c);
      }
    } else {
      int need = (nblk + bpc - 1) / bpc;
      if (int(free_chunks.size()) - need < cfg.kv_reserve_chunks)
        return fail(HARLI_ERR_OOM, "pool: %d tensor chunks would eat the KV reserve", need);
      int run = 0, prev = -2;
      for (int fc : free_chunks) {
        run = (fc == prev + 1) ? run + 1 : 1;
        prev = fc;
        if (run == need) {
          c = fc - need + 1;
          break;
        }
      }
      if (c < 0) return fail(HARLI_ERR_OOM, "pool: no run of %d adjacent free chunks", need);
      for (int i = 0; i < need; ++i) take_chunk_for_tensor(c + i);
    }
    mark_blocks(c, b0, nblk);
    out->cls = HARLI_CLS_TENSOR;
    out->page = -1;
    out->offset = chunk_base(c) + size_t(b0) * cfg.block_bytes;
    out->bytes = size_t(nblk) * cfg.block_bytes;
    out->ptr = slab + out->offset;
    live[out->offset] = Live{HARLI_CLS_TENSOR, out->bytes, requested};
    requested_live += requested;
    reserved_live += out->bytes;
    return HARLI_OK;
  }

  void release_tensor(size_t off, size_t nbytes) {
    size_t first = (off - cfg.small_pool_bytes) / cfg.block_bytes;
    size_t nblk = nbytes / cfg.block_bytes;
    int c_lo = int(first / bpc), c_hi = int((first + nblk - 1) / bpc);
    for (size_t i = 0; i < nblk; ++i) bits[(first + i) / bpc].clr(int((first + i) % bpc));
    tensor_blocks_live -= int64_t(nblk);
    for (int c = c_lo; c <= c_hi; ++c)
      if (bits[c].used == 0) {
        tensor_chunks.erase(c);
        cls[c] = C_FREE;
        free_chunks.insert(c);
      }
  }

  // ---- small tensors: buddy --------------------------------------------------------
  harli_status alloc_small(size_t nbytes, harli_alloc* out) {
    int order = 0;
    while ((cfg.small_granule << order) < nbytes) ++order;
    for (int o = order; o <= max_order; ++o) {
      if (buddy[o].empty()) continue;
      size_t off = *buddy[o].begin();
      buddy[o].erase(buddy[o].begin());
      while (o > order) {  // split, keep the lower half
        --o;
        buddy[o].insert(off + (cfg.small_granule << o));
      }
      out->cls = HARLI_CLS_SMALL;
      out->page = -1;
      out->offset = off;
      out->bytes = cfg.small_granule << order;
      out->ptr = slab + off;
      live[off] = Live{HARLI_CLS_SMALL, out->bytes, nbytes};
      small_bytes_live += out->bytes;
      requested_live += nbytes;
      reserved_live += out->bytes;
      return HARLI_OK;
    }
    harli_status st = alloc_tensor(cfg.block_bytes, nbytes, out);  // pool exhausted: one general block
    if (st == HARLI_OK) ++small_fallbacks;
    return st;
  }

  void release_small(size_t off, size_t nbytes) {
    int o = 0;
    while ((cfg.small_granule << o) < nbytes) ++o;
    small_bytes_live -= nbytes;
    while (o < max_order) {
      size_t bud = off ^ (cfg.small_granule << o);
      auto it = buddy[o].find(bud);
      if (it == buddy[o].end()) break;
      buddy[o].erase(it);
      off = off < bud ? off : bud;
      ++o;
    }
    buddy[o].insert(off);
  }

  void release(size_t off) {
    auto it = live.find(off);
    Live l = it->second;
    live.erase(it);
    requested_live -= l.requested;
    reserved_live -= l.bytes;
    if (l.cls == HARLI_CLS_SMALL)
      release_small(off, l.bytes);
    else
      release_tensor(off, l.bytes);
  }

  // ---- deferred frees -----------------------------------------------------------------
  void poll() {
    size_t k = 0;
    void* seen = nullptr;  // entries that share an event (the pages of one free call) sit next to each other
    int seen_done = 0;
    std::vector<void*> destroy;
    for (size_t i = 0; i < pending.size(); ++i) {
      Pending& p = pending[i];
      if (p.event != seen) seen = p.event, seen_done = event_done(p.event);
      // Only a completed event releases memory.  A query that fails says nothing about the work that still reads
      // the buffer, so the entry stays pending (the memory is held back until the pool is destroyed rather than
      // handed to a second owner).
      if (seen_done > 0) {
        if (p.own) destroy.push_back(p.event);  // after the pass: later entries may share it
        if (p.is_page)
          release_page(p.page);
        else
          release(p.offset);
      } else {
        pending[k++] = p;
      }
    }
    pending.resize(k);
    for (void* e : destroy) event_destroy(e);
  }
};

namespace harli {
void pool_retain(harli_pool* p) {
  if (p) p->refs.fetch_add(1, std::memory_order_relaxed);
}
void pool_release(harli_pool* p) {
  if (!p || p->refs.fetch_sub(1, std::memory_order_acq_rel) != 1) return;
  for (const Pending& q : p->pending)
    if (q.own) event_destroy(q.event);
  delete p;
}
}  // namespace harli

extern "C" {

const char* harli_status_str(harli_status s) {
  switch (s) {
    case HARLI_OK: return "ok";
    case HARLI_ERR_INVALID: return "invalid argument";
    case HARLI_ERR_OOM: return "out of memory";
    case HARLI_ERR_STATE: return "invalid state";
    case HARLI_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* harli_last_error(void) { return g_err.c_str(); }
const char* harli_version(void) { return "harli-mi355x 0.1 (gfx950)"; }

harli_status harli_pool_create(void* slab, size_t slab_bytes, const harli_pool_cfg* cfg, harli_pool** out) {
  if (!cfg || !out) return fail(HARLI_ERR_INVALID, "pool_create: null argument");
  if (cfg->block_bytes == 0 || cfg->small_granule == 0 || cfg->n_layers <= 0 || cfg->page_tokens <= 0 ||
      cfg->kv_row_bytes == 0 || cfg->kv_reserve_chunks < 0)
    return fail(HARLI_ERR_INVALID, "pool_create: zero or negative field in cfg");
  size_t ratio = cfg->block_bytes / cfg->small_granule;
  if (ratio * cfg->small_granule != cfg->block_bytes || (ratio & (ratio - 1)) != 0)
    return fail(HARLI_ERR_INVALID, "pool_create: block_bytes must be small_granule * 2^k");
  if (cfg->small_pool_bytes % cfg->block_bytes != 0)
    return fail(HARLI_ERR_INVALID, "pool_create: small_pool_bytes must be a multiple of block_bytes");
  size_t page_bytes = size_t(cfg->page_tokens) * cfg->kv_row_bytes;
  if (page_bytes > cfg->block_bytes)
    return fail(HARLI_ERR_INVALID, "pool_create: a %zu-byte page does not fit a %zu-byte block", page_bytes,
                cfg->block_bytes);
  size_t chunk_bytes = size_t(cfg->n_layers) * 2 * cfg->block_bytes;
  if (slab_bytes < cfg->small_pool_bytes + chunk_bytes)
    return fail(HARLI_ERR_INVALID, "pool_create: slab of %zu bytes holds no chunk (%zu + %zu needed)", slab_bytes,
                cfg->small_pool_bytes, chunk_bytes);
  size_t n_chunks = (slab_bytes - cfg->small_pool_bytes) / chunk_bytes;
  size_t ppb = cfg->block_bytes / page_bytes;
  if (n_chunks * ppb > size_t(INT32_MAX)) return fail(HARLI_ERR_INVALID, "pool_create: too many pages for int32 ids");
  harli_pool* p = new harli_pool;
  p->slab = static_cast<char*>(slab);
  p->slab_bytes = slab_bytes;
  p->cfg = *cfg;
  p->page_bytes = page_bytes;
  p->chunk_bytes = chunk_bytes;
  p->ppb = int(ppb);
  p->bpc = 2 * cfg->n_layers;
  p->n_chunks = int(n_chunks);
  p->max_order = 0;
  while ((size_t(1) << p->max_order) < ratio) ++p->max_order;
  p->cls.assign(n_chunks, C_FREE);
  p->bits.resize(n_chunks);
  for (int c = 0; c < p->n_chunks; ++c) p->free_chunks.insert(c);
  p->buddy.resize(p->max_order + 1);
  for (size_t a = 0; a < cfg->small_pool_bytes / cfg->block_bytes; ++a)
    p->buddy[p->max_order].insert(a * cfg->block_bytes);
  *out = p;
  return HARLI_OK;
}

void harli_pool_destroy(harli_pool* p) { harli::pool_release(p); }

harli_status harli_pool_alloc(harli_pool* p, harli_class cls, size_t n, harli_alloc* out) {
  if (!p || !out) return fail(HARLI_ERR_INVALID, "pool_alloc: null argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  harli_alloc a{};
  harli_status st;
  switch (cls) {
    case HARLI_CLS_KV_PAGE: {
      int32_t page;
      st = p->alloc_page(&page);
      if (st != HARLI_OK) return st;
      a.cls = HARLI_CLS_KV_PAGE;
      a.page = page;
      a.offset = 0;
      a.bytes = p->page_bytes * size_t(p->bpc);
      a.ptr = nullptr;
      break;
    }
    case HARLI_CLS_AUTO:
      if (n == 0) return fail(HARLI_ERR_INVALID, "pool_alloc: zero bytes");
      st = n < p->cfg.block_bytes ? p->alloc_small(n, &a) : p->alloc_tensor(n, n, &a);
      if (st != HARLI_OK) return st;
      break;
    case HARLI_CLS_TENSOR:
      if (n == 0) return fail(HARLI_ERR_INVALID, "pool_alloc: zero bytes");
      st = p->alloc_tensor(n, n, &a);
      if (st != HARLI_OK) return st;
      break;
    case HARLI_CLS_SMALL:
      if (n == 0 || n >= p->cfg.block_bytes)
        return fail(HARLI_ERR_INVALID, "pool_alloc: SMALL needs 0 < n < block_bytes, got %zu", n);
      st = p->alloc_small(n, &a);
      if (st != HARLI_OK) return st;
      break;
    default:
      return fail(HARLI_ERR_INVALID, "pool_alloc: unknown class %d", int(cls));
  }
  *out = a;
  return HARLI_OK;
}

harli_status harli_pool_alloc_pages(harli_pool* p, int32_t n_pages, int32_t* page_ids) {
  if (!p || (n_pages > 0 && !page_ids) || n_pages < 0) return fail(HARLI_ERR_INVALID, "pool_alloc_pages: bad argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  for (int32_t i = 0; i < n_pages; ++i) {
    harli_status st = p->alloc_page(&page_ids[i]);
    if (st != HARLI_OK) {
      for (int32_t j = i - 1; j >= 0; --j) p->release_page(page_ids[j]);  // all or nothing
      return st;
    }
  }
  return HARLI_OK;
}

// `own`: the pool destroys the event once it has completed.  The pending entry is made with that flag under the
// lock that adds it: a poll from another thread may run as soon as the lock is dropped.
static harli_status free_pages_impl(harli_pool* p, int32_t n_pages, const int32_t* page_ids, void* event, bool own);

static harli_status free_impl(harli_pool* p, const harli_alloc* a, void* event, bool own) {
  if (!p || !a) return fail(HARLI_ERR_INVALID, "pool_free: null argument");
  if (a->cls == HARLI_CLS_KV_PAGE) return free_pages_impl(p, 1, &a->page, event, own);
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  auto it = p->live.find(a->offset);
  if (it == p->live.end()) return fail(HARLI_ERR_INVALID, "pool_free: offset %zu is not a live allocation", a->offset);
  for (const Pending& q : p->pending)
    if (!q.is_page && q.offset == a->offset) return fail(HARLI_ERR_INVALID, "pool_free: offset %zu freed twice", a->offset);
  if (event)
    p->pending.push_back(Pending{event, own, false, -1, a->offset});
  else
    p->release(a->offset);
  return HARLI_OK;
}

harli_status harli_pool_free(harli_pool* p, const harli_alloc* a, void* event) { return free_impl(p, a, event, false); }

harli_status harli_pool_free_pages(harli_pool* p, int32_t n_pages, const int32_t* page_ids, void* event) {
  return free_pages_impl(p, n_pages, page_ids, event, false);
}

static harli_status free_pages_impl(harli_pool* p, int32_t n_pages, const int32_t* page_ids, void* event, bool own) {
  if (!p || (n_pages > 0 && !page_ids) || n_pages < 0) return fail(HARLI_ERR_INVALID, "pool_free_pages: bad argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  for (int32_t i = 0; i < n_pages; ++i) {
    harli_status st = p->check_page(page_ids[i]);
    if (st != HARLI_OK) return st;
    for (int32_t j = 0; j < i; ++j)
      if (page_ids[j] == page_ids[i]) return fail(HARLI_ERR_INVALID, "pool_free_pages: page %d listed twice", page_ids[i]);
    for (const Pending& q : p->pending)
      if (q.is_page && q.page == page_ids[i]) return fail(HARLI_ERR_INVALID, "pool_free_pages: page %d freed twice", page_ids[i]);
  }
  for (int32_t i = 0; i < n_pages; ++i) {
    if (event)
      p->pending.push_back(Pending{event, own && i == 0, true, page_ids[i], 0});  // one entry owns a shared event
    else
      p->release_page(page_ids[i]);
  }
  return HARLI_OK;
}

harli_status harli_pool_kv_addr(const harli_pool* p, int32_t page, int32_t layer, int32_t kv, size_t* byte_off) {
  if (!p || !byte_off) return fail(HARLI_ERR_INVALID, "pool_kv_addr: null argument");
  if (page < 0 || page >= p->n_chunks * p->ppb || layer < 0 || layer >= p->cfg.n_layers || (kv != 0 && kv != 1))
    return fail(HARLI_ERR_INVALID, "pool_kv_addr: (page %d, layer %d, kv %d) out of range", page, layer, kv);
  int c = page / p->ppb, slot = page % p->ppb;
  *byte_off = p->chunk_base(c) + size_t(2 * layer + kv) * p->cfg.block_bytes + size_t(slot) * p->page_bytes;
  return HARLI_OK;
}

harli_status harli_pool_stats(harli_pool* p, harli_pool_stats_t* out) {
  if (!p || !out) return fail(HARLI_ERR_INVALID, "pool_stats: null argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  harli_pool_stats_t s{};
  s.n_chunks = p->n_chunks;
  s.free_chunks = int32_t(p->free_chunks.size());
  s.tensor_chunks = int32_t(p->tensor_chunks.size());
  s.kv_chunks = s.n_chunks - s.free_chunks - s.tensor_chunks;
  s.pages_per_block = p->ppb;
  s.blocks_per_chunk = p->bpc;
  s.kv_pages_live = p->kv_pages_live;
  s.tensor_blocks_live = p->tensor_blocks_live;
  s.small_bytes_live = p->small_bytes_live;
  s.requested_bytes_live = p->requested_live;
  s.reserved_bytes_live = p->reserved_live;
  s.small_fallbacks = p->small_fallbacks;
  s.pending_frees = int64_t(p->pending.size());
  *out = s;
  return HARLI_OK;
}

// ---- inter-task memory coordination (Sec. 4.4) ----
harli_status harli_pool_reserve_chunks_for(const harli_pool* p, double release_time, double slo, int32_t max_bs, int32_t* chunks) {
  if (!p || !chunks || !(release_time >= 0.0) || !(slo > 0.0) || max_bs < 1 || !std::isfinite(release_time) || !std::isfinite(slo))
    return fail(HARLI_ERR_INVALID, "pool_reserve_chunks_for: bad argument");
  // decode steps that pass while the finetune task is still releasing; each of max_bs sequences appends a token
  // per step and may need ceil(steps / page_tokens) new pages in that window
  const double st = std::ceil(release_time / slo - 1e-12);
  if (st > 1e9) return fail(HARLI_ERR_INVALID, "pool_reserve_chunks_for: %.3g decode steps is out of range", st);
  const long long steps = (long long)st;
  const long long pages = (long long)max_bs * ((steps + p->cfg.page_tokens - 1) / p->cfg.page_tokens);
  *chunks = (int32_t)((pages + p->ppb - 1) / p->ppb);
  return HARLI_OK;
}

harli_status harli_pool_set_reserve(harli_pool* p, int32_t chunks) {
  if (!p || chunks < 0) return fail(HARLI_ERR_INVALID, "pool_set_reserve: bad argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->cfg.kv_reserve_chunks = chunks;
  return HARLI_OK;
}

harli_status harli_pool_pressure(harli_pool* p, int32_t* chunks_to_release) {
  if (!p || !chunks_to_release) return fail(HARLI_ERR_INVALID, "pool_pressure: null argument");
  std::lock_guard<std::mutex> lk(p->mu);
  p->poll();
  const int shortfall = std::max(0, p->cfg.kv_reserve_chunks - int(p->free_chunks.size()));
  *chunks_to_release = std::min(shortfall, int(p->tensor_chunks.size()));
  return HARLI_OK;
}

void* harli_pool_slab(const harli_pool* p) { return p->slab; }
size_t harli_pool_slab_bytes(const harli_pool* p) { return p->slab_bytes; }
void harli_pool_geom(const harli_pool* p, harli::KvGeom* g) {
  g->small_pool_bytes = p->cfg.small_pool_bytes;
  g->chunk_bytes = p->chunk_bytes;
  g->block_bytes = p->cfg.block_bytes;
  g->page_bytes = p->page_bytes;
  g->row_bytes = p->cfg.kv_row_bytes;
  g->pages_per_block = p->ppb;
  g->page_tokens = p->cfg.page_tokens;
  g->n_layers = p->cfg.n_layers;
  g->n_pages_total = p->n_chunks * p->ppb;
}

}  // extern "C"

namespace harli {
// Release whose event the pool takes ownership of (library-internal: the finetune unit records
// one event per released buffer and cannot know when the pool will have polled it).
harli_status pool_free_owned(harli_pool* p, const harli_alloc* a, void* event) {
  if (!event) return harli_pool_free(p, a, nullptr);
  harli_status st = free_impl(p, a, event, true);
  if (st != HARLI_OK) event_destroy(event);
  return st;
}
}  // namespace harli
