// Host-side stress of the library's CPU logic, built by tests/test_sanitizers.py under -fsanitize=address,undefined and,
// with the argument "threads", under -fsanitize=thread: the unified pool (Harli Sec. 4.2-4.5), the latency predictor and
// runtime scheduler (Sec. 5, Sec. 6) and the weight-window plan (Sec. 4.3).  It links pool.cpp and sched.cpp as they
// are (no GPU call is made: events are the integers below) and checks the invariants a shadow model can state
// cheaply: live allocations never overlap, statistics add up, everything returns to FREE, predictions are finite.
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <random>
#include <thread>
#include <vector>

#include "harli.h"
#include "harli_sched.h"
#include "window_plan.h"

// The pool asks these two about the events it was given; here an event is a pointer to an int that the test flips.
namespace harli {
int event_done(void* e) { return *static_cast<std::atomic<int>*>(e) != 0 ? 1 : 0; }
void event_destroy(void*) {}
}  // namespace harli

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: CHECK(%s) failed: %s\n", __FILE__, __LINE__, #cond, harli_last_error()); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

static harli_pool* make_pool(int n_chunks, int reserve, char** slab_out) {
  harli_pool_cfg cfg{};
  cfg.block_bytes = 64 << 10;
  cfg.n_layers = 2;
  cfg.page_tokens = 16;
  cfg.kv_row_bytes = 256;
  cfg.small_pool_bytes = 4 * cfg.block_bytes;
  cfg.small_granule = 2 << 10;
  cfg.kv_reserve_chunks = reserve;
  const size_t chunk = size_t(cfg.n_layers) * 2 * cfg.block_bytes;
  const size_t bytes = cfg.small_pool_bytes + size_t(n_chunks) * chunk;
  char* slab = reinterpret_cast<char*>(uintptr_t(1) << 40);  // an address only: the pool never dereferences it
  harli_pool* p = nullptr;
  CHECK(harli_pool_create(slab, bytes, &cfg, &p) == HARLI_OK);
  *slab_out = slab;
  return p;
}

// ---- one thread, random trace against a shadow model ----------------------------------------------------------------
static void pool_trace(unsigned seed, int ops) {
  char* slab;
  harli_pool* p = make_pool(24, 2, &slab);
  std::mt19937 rng(seed);
  struct Live {
    harli_alloc a;
  };
  std::vector<Live> live;
  std::vector<int32_t> pages;
  std::map<size_t, size_t> ranges;  // offset -> end of live TENSOR / SMALL allocations
  std::vector<std::atomic<int>*> events;
  std::vector<size_t> deferred;  // offsets freed behind an event that has not fired
  auto overlap_free = [&](size_t off, size_t n) {
    auto it = ranges.upper_bound(off);
    if (it != ranges.end() && it->first < off + n) return false;
    if (it != ranges.begin() && std::prev(it)->second > off) return false;
    return true;
  };
  for (int i = 0; i < ops; ++i) {
    const int op = rng() % 8;
    if (op < 3) {  // tensor or small allocation
      const bool small = rng() & 1;
      const size_t n = small ? 1 + rng() % (60 << 10) : (size_t(1) + rng() % 5) * (48 << 10);
      harli_alloc a{};
      const harli_status s = harli_pool_alloc(p, HARLI_CLS_AUTO, n, &a);
      if (s == HARLI_OK) {
        CHECK(a.bytes >= n && a.ptr == slab + a.offset);
        CHECK(overlap_free(a.offset, a.bytes));
        ranges[a.offset] = a.offset + a.bytes;
        live.push_back({a});
      } else {
        CHECK(s == HARLI_ERR_OOM);
      }
    } else if (op == 3) {  // a few KV pages
      int32_t ids[5];
      const int n = 1 + rng() % 5;
      const harli_status s = harli_pool_alloc_pages(p, n, ids);
      if (s == HARLI_OK) {
        for (int k = 0; k < n; ++k) {
          size_t off = 0;
          CHECK(harli_pool_kv_addr(p, ids[k], 1, 1, &off) == HARLI_OK);
          pages.push_back(ids[k]);
        }
      } else {
        CHECK(s == HARLI_ERR_OOM);
      }
    } else if (op < 6 && !live.empty()) {  // free, half of them behind an event that fires later
      const size_t k = rng() % live.size();
      std::atomic<int>* ev = nullptr;
      if (rng() & 1) events.push_back(ev = new std::atomic<int>(0));
      CHECK(harli_pool_free(p, &live[k].a, ev) == HARLI_OK);
      CHECK(harli_pool_free(p, &live[k].a, nullptr) == HARLI_ERR_INVALID);  // double free is refused
      if (!ev) ranges.erase(live[k].a.offset);
      else deferred.push_back(live[k].a.offset);  // stays occupied in the shadow until its event fires: the pool must
      live[k] = live.back();                      // not hand the range to anyone before that
      live.pop_back();
    } else if (op == 6 && !pages.empty()) {
      const size_t k = rng() % pages.size();
      CHECK(harli_pool_free_pages(p, 1, &pages[k], nullptr) == HARLI_OK);
      pages[k] = pages.back();
      pages.pop_back();
    } else {  // fire every outstanding event
      for (auto* e : events) e->store(1);
      for (size_t off : deferred) ranges.erase(off);
      deferred.clear();
    }
    harli_pool_stats_t st{};
    CHECK(harli_pool_stats(p, &st) == HARLI_OK);
    CHECK(st.free_chunks + st.kv_chunks + st.tensor_chunks == st.n_chunks);
    CHECK(st.kv_pages_live == (int64_t)pages.size());
    CHECK(st.reserved_bytes_live >= st.requested_bytes_live);
  }
  for (auto* e : events) e->store(1);
  for (auto& l : live) CHECK(harli_pool_free(p, &l.a, nullptr) == HARLI_OK);
  if (!pages.empty()) CHECK(harli_pool_free_pages(p, (int32_t)pages.size(), pages.data(), nullptr) == HARLI_OK);
  harli_pool_stats_t st{};
  CHECK(harli_pool_stats(p, &st) == HARLI_OK);
  CHECK(st.pending_frees == 0 && st.free_chunks == st.n_chunks && st.small_bytes_live == 0 && st.tensor_blocks_live == 0);
  harli_pool_destroy(p);
  for (auto* e : events) delete e;
}

static void sched_trace(unsigned seed) {
  std::mt19937 rng(seed);
  std::uniform_real_distribution<double> noise(0.97, 1.03);
  const int L = 10;
  harli_predictor* p = nullptr;
  CHECK(harli_pred_create(L, &p) == HARLI_OK);
  for (int lv = 1; lv <= L; ++lv)
    for (int k = 0; k < 12; ++k) {
      const int bs = 1 + rng() % 64, sl = 128 + rng() % 4000;
      const double lat = (bs * 0.02 + 1.0 + bs * 1e-5 * sl) * (1.0 + 2.0 / lv) * noise(rng);
      CHECK(harli_pred_add_solo(p, lv, bs, sl, lat) == HARLI_OK);
    }
  for (int i = 1; i < L; ++i)
    for (int f = 1; i + f <= L; ++f) CHECK(harli_pred_add_colo(p, i, f, (0.9 + 0.05 * i + 0.08 * f) * noise(rng), 1.0) == HARLI_OK);
  CHECK(harli_pred_add_solo(p, 0, 1, 1, 1.0) == HARLI_ERR_INVALID);
  CHECK(harli_pred_fit(p) == HARLI_OK);
  for (int floor = 1; floor >= 0; --floor) {
    CHECK(harli_pred_set_colo_floor(p, floor) == HARLI_OK);
    CHECK(harli_pred_fit(p) == HARLI_OK);
    for (int k = 0; k < 200; ++k) {
      const int i = 1 + rng() % (L - 1), f = 1 + rng() % (L - i), bs = 1 + rng() % 256, sl = 1 + rng() % 8192;
      double a = 0, b = 0;
      CHECK(harli_pred_solo(p, i, bs, sl, &a) == HARLI_OK && std::isfinite(a));
      CHECK(harli_pred_colo(p, i, f, bs, sl, &b) == HARLI_OK && std::isfinite(b));
      if (floor) CHECK(b >= a * (1.0 - 1e-12));
    }
  }
  CHECK(harli_pred_set_colo_floor(p, 1) == HARLI_OK);
  CHECK(harli_pred_fit(p) == HARLI_OK);
  harli_scheduler* s = nullptr;
  CHECK(harli_sched_create(p, 40.0, 8, &s) == HARLI_OK);
  for (int k = 0; k < 500; ++k) {
    harli_sched_decision d{};
    const int bs = 1 + rng() % 300, sl = 1 + rng() % 9000;
    CHECK(harli_sched_step(s, bs, sl, rng() % 4 != 0, &d) == HARLI_OK);
    CHECK(d.infer_level >= 1 && d.infer_level <= L && d.ft_level >= 0 && d.infer_level + d.ft_level <= L);
    if (k % 7 == 0) CHECK(harli_pred_observe(p, d.infer_level, 10.0, 10.0 * noise(rng), 1.0) == HARLI_OK);
  }
  harli_sched_destroy(s);
  harli_pred_destroy(p);
}

static void window_trace(unsigned seed) {
  std::mt19937 rng(seed);
  for (int rep = 0; rep < 50; ++rep) {
    const int L = 1 + rng() % 40, n = 1 + rng() % (2 * L);
    harli::WindowPlan w;
    w.init(L, n);
    int item = 0;
    for (int use = 0; use < 6 * L; ++use) {
      if (rng() % 11 == 0) item = rng() % w.items();  // out-of-order use
      int s = w.find(item);
      if (s < 0) {
        s = w.victim(item);
        CHECK(s >= 0 && s < n);
        w.slot_item[s] = item;
      }
      const int nxt = w.refill_after(item);
      if (nxt >= 0) {
        CHECK(w.find(nxt) < 0 && nxt < w.items());
        w.slot_item[s] = nxt;
      }
      for (int a = 0; a < n; ++a)
        for (int b = a + 1; b < n; ++b) CHECK(w.slot_item[a] < 0 || w.slot_item[a] != w.slot_item[b]);
      const std::vector<int> want = w.wanted_items(item, n);
      CHECK((int)want.size() == (n < w.items() ? n : w.items()));
      item = (item + 1) % w.items();
    }
    int calm = 0, slots = n;
    for (int k = 0; k < 40; ++k) {
      const harli::WindowAdvice a = harli::advise_slots(slots, 2 * L, 1 + rng() % 3, rng() % 64, rng() % 64, rng() % 5 == 0, calm);
      CHECK(a.target >= 1 && a.target <= (slots > 2 * L ? slots : 2 * L));
      slots = a.target;
      calm = a.calm;
    }
  }
}

// ---- two threads on one pool: allocations and frees interleave; every thread checks its own allocations ----------
static void thread_body(harli_pool* p, unsigned seed, std::atomic<int>* bad) {
  std::mt19937 rng(seed);
  std::vector<harli_alloc> mine;
  std::vector<int32_t> pages;
  for (int i = 0; i < 4000; ++i) {
    const int op = rng() % 4;
    if (op == 0) {
      harli_alloc a{};
      if (harli_pool_alloc(p, HARLI_CLS_AUTO, 1 + rng() % (200 << 10), &a) == HARLI_OK) mine.push_back(a);
    } else if (op == 1) {
      int32_t id;
      if (harli_pool_alloc_pages(p, 1, &id) == HARLI_OK) pages.push_back(id);
    } else if (op == 2 && !mine.empty()) {
      if (harli_pool_free(p, &mine.back(), nullptr) != HARLI_OK) bad->fetch_add(1);
      mine.pop_back();
    } else if (!pages.empty()) {
      if (harli_pool_free_pages(p, 1, &pages.back(), nullptr) != HARLI_OK) bad->fetch_add(1);
      pages.pop_back();
    }
    harli_pool_stats_t st{};
    if (harli_pool_stats(p, &st) != HARLI_OK) bad->fetch_add(1);
  }
  for (auto& a : mine)
    if (harli_pool_free(p, &a, nullptr) != HARLI_OK) bad->fetch_add(1);
  for (int32_t id : pages)
    if (harli_pool_free_pages(p, 1, &id, nullptr) != HARLI_OK) bad->fetch_add(1);
}

int main(int argc, char** argv) {
  if (argc > 1 && std::strcmp(argv[1], "threads") == 0) {
    char* slab;
    harli_pool* p = make_pool(32, 1, &slab);
    std::atomic<int> bad{0};
    std::thread t1(thread_body, p, 11u, &bad), t2(thread_body, p, 29u, &bad);
    t1.join();
    t2.join();
    CHECK(bad.load() == 0);
    harli_pool_stats_t st{};
    CHECK(harli_pool_stats(p, &st) == HARLI_OK);
    CHECK(st.free_chunks == st.n_chunks && st.small_bytes_live == 0 && st.kv_pages_live == 0);
    harli_pool_destroy(p);
    std::puts("threads ok");
    return 0;
  }
  for (unsigned seed = 1; seed <= 6; ++seed) pool_trace(seed, 4000);
  for (unsigned seed = 1; seed <= 3; ++seed) sched_trace(seed);
  for (unsigned seed = 1; seed <= 3; ++seed) window_trace(seed);
  std::puts("traces ok");
  return 0;
}
