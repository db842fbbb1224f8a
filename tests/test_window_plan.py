"""Window over the finetune task's frozen weights (Sec. 4.3), host logic only (CPU).

The CPU model is pinned by what the policy must guarantee whatever its code looks like: a training step that walks
the weights in their fixed order never waits for a copy once the window is primed; up to LOOKAHEAD slots it loads
exactly one copy per use (2L per step) and always has the next n - 1 copies on the device; a larger window has the
next LOOKAHEAD - 1 copies on the device, copies (2L - n) * 2L / (2L - LOOKAHEAD) items per step and stays within a
small factor of the best any eviction rule could do (brute force); a window that covers the whole cycle never copies.  The library's plan is then compared with the model access by access, on the regular order and on random
ones."""
import numpy as np
import pytest

from oracle import window_model as WM
from paper_2511_11729_amd import binding as hb


def step_order(L):
    return [WM.item_of(l, False, L) for l in range(L)] + [WM.item_of(l, True, L) for l in range(L - 1, -1, -1)]


def test_item_numbering_follows_the_order_of_use():
    L = 5
    assert step_order(L) == list(range(2 * L))
    assert WM.item_of(0, True, L) == 2 * L - 1 and WM.item_of(L - 1, True, L) == L and WM.item_of(L - 1, False, L) == L - 1


@pytest.mark.parametrize("L,n", [(4, 1), (4, 2), (4, 3), (6, 4), (8, 4), (3, 4), (32, 3)])
def test_regular_steps_never_miss_and_load_one_copy_per_use(L, n):
    w = WM.Window(L, n)
    order = step_order(L) * 3
    loads = 0
    for k, it in enumerate(order):
        resident_before = set(w.slots)
        # the item itself and the next n - 1 in the order are on the device when the item is used
        for d in range(min(n, 2 * L)):
            assert (it + d) % (2 * L) in resident_before, (k, it, d)
        s, miss, refill = w.access(it)
        assert miss == -1
        assert refill == (it + n) % (2 * L)                    # "the first layer outside the window"
        assert len(set(w.slots)) == n and it not in w.slots    # the used copy was evicted, no duplicates
        loads += 1
    assert loads == len(order)


def _optimal_loads(N, n, cycles):
    """Fewest on-demand loads any eviction rule can have on the cyclic order (evict the item used farthest ahead)."""
    res, loads = list(range(n)), 0
    for t in range(N * cycles):
        it = t % N
        if it not in res:
            loads += 1
            far = max(res, key=lambda x: (x - it) % N)
            res[res.index(far)] = it
    return loads


@pytest.mark.parametrize("L,n", [(4, 5), (4, 7), (6, 5), (3, 5), (32, 6), (32, 40), (32, 56), (32, 63)])
def test_large_windows_keep_what_is_not_needed_soon(L, n):
    N, K = 2 * L, WM.LOOKAHEAD
    w = WM.Window(L, n)
    cycles = 4 * (N - K)
    loads_by_cycle = []
    for c in range(cycles):
        loads = 0
        for it in range(N):
            before = set(w.slots)
            for d in range(K):                                   # the item and the next K - 1 are on the device
                assert (it + d) % N in before, (c, it, d)
            s, miss, refill = w.access(it)
            assert miss == -1
            assert refill in (-1, (it + K) % N)                  # a copy always starts K uses before its item is needed
            assert len(set(w.slots)) == n
            loads += refill >= 0
        loads_by_cycle.append(loads)
    if 2 * (N - n) <= N - K:                                     # the copies of a step are spread out, never back to back
        w2, last, gaps = WM.Window(L, n), None, []
        for t in range(6 * N):
            if w2.access(t % N)[2] >= 0:
                if last is not None:
                    gaps.append(t - last)
                last = t
        assert min(gaps) >= (N - K) // (N - n) - 1 >= 1
    steady = loads_by_cycle[N - K:]                              # the pattern repeats every 2L - K steps
    assert sum(steady[: N - K]) == N * (N - n)
    assert sum(steady) * (N - K) == len(steady) * N * (N - n)
    # against the best possible (which needs no slot for copies in flight): never better, and close for wide windows
    best = _optimal_loads(N, n, cycles) / cycles
    mine = sum(steady) / len(steady)
    assert mine >= best - 1e-9
    if n >= 4 * K:                                               # windows much wider than the prefetch distance
        assert mine <= 1.15 * best


@pytest.mark.parametrize("L,n", [(4, 8), (4, 11), (1, 2)])
def test_a_window_over_the_whole_cycle_never_copies(L, n):
    w = WM.Window(L, min(n, 2 * L))
    for it in step_order(L) * 2:
        assert w.access(it)[1:] == (-1, -1)
    assert sorted(w.slots) == list(range(2 * L))


def test_out_of_order_use_is_served_on_demand_and_the_window_recovers():
    L, n = 6, 3
    w = WM.Window(L, n)
    assert w.access(0) == (0, -1, 3)            # regular start: slots hold 3, 1, 2
    s, miss, refill = w.access(9)               # a jump: 9 is absent; of 3, 1, 2 the one farthest ahead of 9 is 3 (6 steps)
    assert (s, miss) == (0, 9) and refill == 10
    assert sorted(w.slots) == [1, 2, 10]
    s, miss, refill = w.access(10)              # resident now
    assert miss == -1 and refill == 11
    # back to the regular walk from 11: at most n - 1 on-demand loads (the stale copies 1 and 2 are replaced), then none
    misses = [w.access(it % 12)[1] for it in range(11, 11 + 24)]
    assert sum(m >= 0 for m in misses[: n]) <= n - 1 and all(m == -1 for m in misses[n:])


@pytest.mark.parametrize("L,n", [(4, 1), (4, 3), (5, 4), (7, 14), (16, 5), (16, 20), (32, 60), (6, 9)])
def test_library_plan_equals_the_model_on_regular_and_random_orders(L, n):
    rng = np.random.default_rng(L * 100 + n)
    seqs = [step_order(L) * 3,
            [int(x) for x in rng.integers(0, 2 * L, 200)],
            step_order(L)[:3] + [int(x) for x in rng.integers(0, 2 * L, 10)] + step_order(L) * 2]
    for seq in seqs:
        w = WM.Window(L, min(n, 2 * L))
        want = [w.access(it) for it in seq]
        slot, miss, refill = hb.dbg_window_plan(L, n, seq)
        assert list(zip(slot, miss, refill)) == want


def test_plan_rejects_bad_arguments():
    for L, n, seq in [(0, 1, [0]), (2, 0, [0]), (2, 1, [4]), (2, 1, [-1])]:
        with pytest.raises(hb.HarliError):
            hb.dbg_window_plan(L, n, seq)


# ---- window size between training steps (Sec. 4.4; step sizes are the library's own, stated in its header) ----
# hand-worked: one slot = 3 chunks, so a group of four slots = 12 chunks
ADVISE_PINS = [
    # slots, max, slot_chunks, free, need, pressed, calm -> target, calm
    ((64, 64, 3, 100, 130, False, 1), (52, 0)),    # 30 chunks short: three groups go
    ((64, 64, 3, 129, 130, False, 0), (60, 0)),    # one chunk short still costs a whole group
    ((64, 64, 3, 500, 130, True, 5), (60, 0)),     # pressed with room: one group, and the calm count starts over
    ((8, 64, 3, 0, 1000, True, 0), (4, 0)),        # never under one group
    ((2, 64, 3, 0, 1000, True, 0), (2, 0)),        # a window under one group is left alone (never grows under pressure)
    ((40, 64, 3, 200, 130, False, 0), (40, 1)),    # first roomy step: wait
    ((40, 64, 3, 200, 130, False, 1), (44, 2)),    # second in a row: one group more
    ((44, 64, 3, 200, 130, False, 2), (48, 3)),    # and one per step after that
    ((62, 64, 3, 200, 130, False, 1), (64, 2)),    # clipped to the largest window
    ((64, 64, 3, 900, 130, False, 7), (64, 0)),    # full: nothing to grow
    ((40, 64, 3, 154, 130, False, 1), (40, 0)),    # exactly need + 8 slots free is not roomy
    ((40, 64, 3, 155, 130, False, 1), (44, 2)),
    ((40, 64, 3, 130, 130, False, 1), (40, 0)),    # just enough: keep
]


@pytest.mark.parametrize("args,want", ADVISE_PINS)
def test_window_size_rule_hand_worked(args, want):
    assert WM.advise_slots(*args) == want
    assert hb.ft_window_advise(*args) == want


def test_window_size_rule_library_equals_model_on_a_replayed_pool():
    """A pool of `total` chunks shared by the window, a training step's activations and a KV cache that swells and
    shrinks: both statements of the rule take the same decisions, the window stays inside its bounds, a shrink frees
    enough for the step unless the window is already at one group, and a calm stretch restores the full window."""
    rng = np.random.default_rng(11)
    for trial in range(20):
        slot_chunks = int(rng.integers(1, 6))
        top = int(rng.choice([8, 24, 64]))
        need = int(rng.integers(20, 120))
        total = top * slot_chunks + need + int(rng.integers(0, 60))
        slots, calm_l, calm_m = top, 0, 0
        kv = 0
        for step in range(300):
            phase = (step // 60) % 3                       # light, heavy, light again
            kv = max(0, min(total, kv + int(rng.integers(-6, 8)) + (10 if phase == 1 else -10)))
            free = max(0, total - slots * slot_chunks - kv)
            pressed = bool(free == 0 or rng.random() < (0.3 if phase == 1 else 0.0))
            t_m, calm_m = WM.advise_slots(slots, top, slot_chunks, free, need, pressed, calm_m)
            t_l, calm_l = hb.ft_window_advise(slots, top, slot_chunks, free, need, pressed, calm_l)
            assert (t_l, calm_l) == (t_m, calm_m)
            assert min(slots, 4) <= t_m <= top
            assert (t_m - slots) % 4 == 0 or t_m in (top, min(slots, 4))        # whole groups, unless clipped
            if t_m < slots and t_m > 4:
                assert free + (slots - t_m) * slot_chunks >= need      # the groups given up cover the shortage
            if t_m > slots:
                assert not pressed and free > need + 8 * slot_chunks
            slots = t_m
        kv = 0
        for step in range(2 + top // 4):                   # empty cache: back to the full window, a group per step
            free = total - slots * slot_chunks
            slots, calm_m = WM.advise_slots(slots, top, slot_chunks, free, need, False, calm_m)
        assert slots == top or total - slots * slot_chunks <= need + 8 * slot_chunks


def test_window_size_rule_rejects_bad_arguments():
    for bad in [(0, 4, 1, 0, 0, False, 0), (8, 4, 1, 0, 0, False, 0), (4, 8, 0, 0, 0, False, 0), (4, 8, 1, -1, 0, False, 0),
                (4, 8, 1, 0, -1, False, 0), (4, 8, 1, 0, 0, False, -1)]:
        with pytest.raises(hb.HarliError) as e:
            hb.ft_window_advise(*bad)
        assert e.value.status == hb.HARLI_ERR_INVALID
