// Residency plan of the window over the finetune task's frozen weights (Harli Sec. 4.3): pure host logic, no HIP.
//
// One training step touches the frozen weights in a fixed cyclic order: the forward copies W of layers 0..L-1, then the
// transposed copies W^T of layers L-1..0 (the backward pass), then the next step's forward again.  Numbering these
// 2L "items" 0..2L-1 in that order, a window of n device slots holds the items about to be used.  After an item has
// been used its slot receives the nearest item among the next min(n, kLookahead) that no slot holds; when all of them
// are on the device the used item simply stays.  With n <= kLookahead this is the paper's sliding window (every use
// evicts the layer just computed and prefetches "the first layer outside the window": 2L copies per step whatever n);
// with more slots only the next kLookahead items are prefetched and the other n - kLookahead slots keep their items,
// so a step copies (2L - n) * 2L / (2L - kLookahead) items on average instead of 2L -- the traffic falls as the window grows, which
// is what makes shrinking and growing the window under memory pressure (Sec. 4.4) a smooth trade.  An item requested
// while absent (out-of-order use, or a window that was just resized) is loaded on demand into an empty slot or,
// failing that, the slot whose item is needed farthest in the future.
#pragma once
#include <vector>

namespace harli {

constexpr int kLookahead = 4;  // uses between the start of a copy and the use of the item (a copy takes 2-3 layer units)

struct WindowPlan {
  int L = 0, n = 0;
  std::vector<int> slot_item;  // item resident (or being loaded) per slot, -1 = empty

  void init(int layers, int slots) {
    L = layers;
    n = slots;
    slot_item.assign(n, -1);
  }
  int items() const { return 2 * L; }
  static int item_of(int layer, bool backward, int layers) { return backward ? 2 * layers - 1 - layer : layer; }
  int find(int item) const {
    for (int s = 0; s < n; ++s)
      if (slot_item[s] == item) return s;
    return -1;
  }
  // how many uses ahead of `from` the item `to` comes (0 = itself)
  int ahead(int from, int to) const { return ((to - from) % items() + items()) % items(); }
  int victim(int item) const {
    int best = -1, far = -1;
    for (int s = 0; s < n; ++s) {
      if (slot_item[s] < 0) return s;
      const int d = ahead(item, slot_item[s]);
      if (d > far) far = d, best = s;
    }
    return best;
  }
  // The items a window of `slots` slots should hold when `first` is the next item used, in order of use: the next
  // kLookahead items, and of the others all but 2L - slots that are spread evenly over the cycle.  The refill rule
  // moves every absent item kLookahead places back per visit, so an even spread stays even; copies then come one at a
  // time with compute in between instead of in one burst that the host link cannot hide.
  std::vector<int> wanted_items(int first, int slots) const {
    const int N = items();
    std::vector<int> out;
    if (slots >= N) {
      for (int d = 0; d < N; ++d) out.push_back((first + d) % N);
      return out;
    }
    if (slots <= kLookahead) {
      for (int d = 0; d < slots; ++d) out.push_back((first + d) % N);
      return out;
    }
    const int m = N - slots;  // absent items: offsets kLookahead + ((2j + 1)(N - kLookahead)) / (2m), distinct since m <= N - kLookahead
    std::vector<char> absent(N, 0);
    for (int j = 0; j < m; ++j) absent[kLookahead + ((2 * j + 1) * (N - kLookahead)) / (2 * m)] = 1;
    for (int d = 0; d < N; ++d)
      if (!absent[d]) out.push_back((first + d) % N);
    return out;
  }
  int refill_after(int item) const {
    const int k = n < kLookahead ? n : kLookahead;
    for (int d = 1; d <= k; ++d) {
      const int cand = (item + d) % items();
      if (cand == item) return -1;
      if (find(cand) < 0) return cand;
    }
    return -1;
  }
};

// ---- Window size between training steps (Sec. 4.4: the finetune task gives memory back when inference needs it
// and takes it again when chunks are free).  The paper states the behaviour, not step sizes; these are this
// library's: slots move in groups of kLookahead (what one refill round covers), the window shrinks at once by as
// many groups as cover the shortage, and grows by one group per step after kCalmSteps steps in a row with more than
// kGrowSlack slots' worth of chunks free beyond the step's own need.
constexpr int kCalmSteps = 2;
constexpr int kGrowSlack = 8;

struct WindowAdvice {
  int target;  // slots to ask harli_ft_window_resize for (== slots: leave the window alone)
  int calm;    // updated count of roomy steps in a row
};

// slots / max_slots: the window now and the most it may hold.  slot_chunks: pool chunks one slot takes.
// free_chunks: chunks free in the pool now.  need_chunks: chunks the next training step and the KV reserve need free.
// pressed: inference asked for memory since the last step (back-pressure, or the last step ran out of memory).
inline WindowAdvice advise_slots(int slots, int max_slots, long long slot_chunks, long long free_chunks, long long need_chunks,
                                 bool pressed, int calm) {
  const long long group = (long long)kLookahead * slot_chunks;
  if (pressed || free_chunks < need_chunks) {
    long long shortage = need_chunks - free_chunks;
    if (shortage < slot_chunks) shortage = slot_chunks;
    const long long groups = (shortage + group - 1) / group;
    const int floor_slots = slots < kLookahead ? slots : kLookahead;  // a window never grows here, nor falls under one group
    long long t = (long long)slots - kLookahead * groups;
    if (t < floor_slots) t = floor_slots;
    return {(int)t, 0};
  }
  if (free_chunks > need_chunks + (long long)kGrowSlack * slot_chunks && slots < max_slots) {
    calm += 1;
    if (calm >= kCalmSteps) {
      const int t = slots + kLookahead < max_slots ? slots + kLookahead : max_slots;
      return {t, calm};
    }
    return {slots, calm};
  }
  return {slots, 0};
}

}  // namespace harli
