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
