"""The synthetic request trace (workloads.make_arrivals) that stands in for the paper's production trace (Sec. 8.1):
seeded, piecewise-constant Poisson arrivals sized by Little's law, log-normal prompts, geometric outputs.  CPU only."""
import numpy as np

import workloads as wl


def test_same_seed_same_trace_and_other_workload_other_trace():
    a = wl.make_arrivals(wl.workload(4), 500)
    b = wl.make_arrivals(wl.workload(4), 500)
    c = wl.make_arrivals(wl.workload(2), 500)
    assert a == b and a != c


def test_rates_follow_the_targets_phase_by_phase():
    targets, mean_out, ph = (4, 64, 16), 32, 4000
    arr = wl.make_arrivals(wl.workload(4), 3 * ph, targets=targets, mean_out=mean_out, phase_steps=ph)
    for k, t in enumerate(targets):
        n = sum(len(r) for r in arr[k * ph:(k + 1) * ph])
        lam = t / mean_out
        assert abs(n - lam * ph) < 5 * np.sqrt(lam * ph)            # Poisson count, five standard deviations


def test_lengths_have_the_stated_distributions():
    arr = wl.make_arrivals(wl.workload(4), 20000, targets=(64,), mean_out=50, prompt=("lognormal", 800, 0.6, 8192))
    reqs = [r for step in arr for r in step]
    p = np.array([r[0] for r in reqs], float)
    o = np.array([r[1] for r in reqs], float)
    assert len(reqs) > 20000
    assert p.min() >= 1 and p.max() <= 8192 and o.min() >= 1
    assert abs(np.median(p) - 800) < 25                             # log-normal: the median is the scale
    assert abs(np.std(np.log(p[p < 8192])) - 0.6) < 0.02
    assert abs(o.mean() - 50) < 1.5                                 # geometric on {1, 2, ...}
    assert abs(np.mean(o == 1) - 1 / 50) < 0.004
    u = wl.make_arrivals(wl.workload(4), 5000, targets=(32,), mean_out=8, prompt=("uniform", 5, 120))
    up = np.array([r[0] for step in u for r in step])
    assert up.min() == 5 and up.max() == 120 and abs(up.mean() - 62.5) < 1.5


def test_steady_state_batch_is_the_target_by_littles_law():
    # a host-only replay of continuous batching with unlimited capacity: every request runs for its output length
    target, mean_out, steps = 24, 40, 30000
    arr = wl.make_arrivals(wl.workload(4), steps, targets=(target,), mean_out=mean_out)
    running, sizes = [], []
    for reqs in arr:
        running.extend(o for _, o in reqs)
        sizes.append(len(running))
        running = [o - 1 for o in running if o > 1]
    assert abs(np.mean(sizes[10 * mean_out:]) - target) < 1.0
