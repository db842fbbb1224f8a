"""CPU model of the window over the finetune task's frozen weights (Harli Sec. 4.3).

TEST INFRASTRUCTURE ONLY: the product path never imports it.  It states the residency policy the library's host
logic (`harli_dbg_window_plan`, and through it `harli_ft_window_*`) is compared with.

The frozen weights of an L-layer model are used, step after step, in the cyclic order
    forward copy of layer 0, 1, ..., L-1, then backward (transposed) copy of layer L-1, ..., 0,
2L "items" numbered in that order.  A window of n slots keeps the next items on the device (the paper: when a layer
has been computed its frozen weights are evicted and those of the first layer outside the window are prefetched):

* access of an item that is resident: hit;
* access of an absent item: it is loaded at once into an empty slot, else into the slot whose item comes latest
  in the cyclic order counted from the accessed item;
* after every access the slot just used is refilled with the nearest absent item among the next min(n, LOOKAHEAD);
  if all of them are present nothing is loaded and the used item stays.  Up to LOOKAHEAD slots this is the paper's
  sliding window (one copy per use).  Reading taken for larger windows: the paper gives the window as the means to
  trade memory for copy traffic (Sec. 4.3, 4.4) without stating a policy for windows much larger than the prefetch
  distance; evicting on every use would copy all 2L items per step whatever the window size, so only the next
  LOOKAHEAD items are prefetched and the remaining slots keep what they hold ((2L - n) * 2L / (2L - LOOKAHEAD) copies per
  step on average).
"""
from __future__ import annotations


LOOKAHEAD = 4


def item_of(layer: int, backward: bool, n_layers: int) -> int:
    return 2 * n_layers - 1 - layer if backward else layer


def wanted_items(n_layers: int, n_slots: int, first: int = 0):
    """What a window of n_slots holds before `first` is used, in order of use: everything if it fits; the next n_slots
    items up to LOOKAHEAD slots (the sliding window); otherwise the next LOOKAHEAD items and, of the rest, all but
    2L - n_slots items spread evenly over the cycle (offset LOOKAHEAD + floor((2j + 1)(2L - LOOKAHEAD) / (2m)) for
    the j-th of the m absent ones).  The refill rule moves an absent item LOOKAHEAD places back each time it comes up,
    so the spread stays even and the copies of a step are never neighbours in the order of use."""
    N = 2 * n_layers
    if n_slots >= N:
        return [(first + d) % N for d in range(N)]
    if n_slots <= LOOKAHEAD:
        return [(first + d) % N for d in range(n_slots)]
    m = N - n_slots
    absent = {LOOKAHEAD + ((2 * j + 1) * (N - LOOKAHEAD)) // (2 * m) for j in range(m)}
    return [(first + d) % N for d in range(N) if d not in absent]


class Window:
    def __init__(self, n_layers: int, n_slots: int, prefill: bool = True):
        self.items = 2 * n_layers
        self.n = n_slots
        self.slots = [-1] * n_slots
        if prefill:
            self.slots = wanted_items(n_layers, min(n_slots, self.items))

    def _ahead(self, frm: int, to: int) -> int:
        return (to - frm) % self.items

    def access(self, item: int):
        """Returns (slot, item loaded on a miss or -1, item loaded into the slot afterwards or -1)."""
        miss = -1
        if item in self.slots:
            s = self.slots.index(item)
        else:
            if -1 in self.slots:
                s = self.slots.index(-1)
            else:
                s = max(range(self.n), key=lambda q: (self._ahead(item, self.slots[q]), -q))
            self.slots[s] = item
            miss = item
        refill = -1
        for d in range(1, min(self.n, LOOKAHEAD) + 1):
            cand = (item + d) % self.items
            if cand == item:
                break
            if cand not in self.slots:
                refill = cand
                break
        if refill >= 0:
            self.slots[s] = refill
        return s, miss, refill


# ---- window size between training steps (Sec. 4.4) ----
# The paper: when inference runs short of memory the finetune task shrinks its window and hands the chunks over; when
# memory is free again the window grows back.  It gives no step sizes.  Reading taken here (the library states the same
# rule in its header): slots move in groups of LOOKAHEAD; under pressure, or when fewer chunks are free than the next
# step needs, the window shrinks at once by as many groups as cover the shortage (at least one slot's worth), but never
# under one group and never upwards; with more than GROW_SLACK slots' worth of chunks free beyond the need, the second
# such step in a row and every one after it adds one group, up to the largest window allowed.
CALM_STEPS = 2
GROW_SLACK = 8


def advise_slots(slots: int, max_slots: int, slot_chunks: int, free_chunks: int, need_chunks: int, pressed: bool, calm: int):
    """Returns (target slots, updated count of roomy steps in a row)."""
    group = LOOKAHEAD * slot_chunks
    if pressed or free_chunks < need_chunks:
        shortage = max(need_chunks - free_chunks, slot_chunks)
        groups = -(-shortage // group)
        return max(min(slots, LOOKAHEAD), slots - LOOKAHEAD * groups), 0
    if free_chunks > need_chunks + GROW_SLACK * slot_chunks and slots < max_slots:
        calm += 1
        if calm >= CALM_STEPS:
            return min(max_slots, slots + LOOKAHEAD), calm
        return slots, calm
    return slots, 0
