"""Pins of the predictor / allocation oracle (CPU only): closed forms, planted coefficients, the normal
equations, the paper's 45 plans, hand-worked choices."""
import itertools

import numpy as np

from oracle import sched_oracle as S


def test_eq1_three_points_equal_the_hand_solution():
    # exactly determined: solve the 3x3 system by Cramer's rule, no library routine
    pts = [(4, 100, 1.30), (16, 100, 2.50), (16, 400, 4.90)]
    def det(m):
        return (m[0][0] * (m[1][1] * m[2][2] - m[1][2] * m[2][1]) - m[0][1] * (m[1][0] * m[2][2] - m[1][2] * m[2][0])
                + m[0][2] * (m[1][0] * m[2][1] - m[1][1] * m[2][0]))
    A = [[bs, 1.0, bs * n] for bs, n, _ in pts]
    y = [p[2] for p in pts]
    D = det(A)
    sol = []
    for c in range(3):
        M = [row[:] for row in A]
        for r in range(3):
            M[r][c] = y[r]
        sol.append(det(M) / D)
    got = S.fit_solo(pts)
    assert np.allclose(got, sol, rtol=1e-10, atol=1e-12)
    # and the model reproduces the points
    for bs, n, lat in pts:
        assert abs(S.predict_solo(got, bs, n) - lat) < 1e-10


def test_eq1_recovers_planted_coefficients_and_is_linear_in_seqlen():
    b0, c0, k0 = 0.0125, 0.9, 3.1e-5
    pts = [(bs, n, bs * b0 + c0 + bs * k0 * n) for bs in (4, 16, 64) for n in (64, 128, 256, 512)]
    got = S.fit_solo(pts)
    assert np.allclose(got, (b0, c0, k0), rtol=1e-9)
    # slope in seqlen at fixed batch is bs*k0; the intercept at bs -> 0 is c0
    assert abs((S.predict_solo(got, 16, 301) - S.predict_solo(got, 16, 300)) - 16 * k0) < 1e-12
    assert abs(S.predict_solo(got, 0, 12345) - c0) < 1e-9


def test_least_squares_satisfies_the_normal_equations():
    rng = np.random.default_rng(7)
    pts = [(bs, n, 0.02 * bs + 1.0 + 2e-5 * bs * n + 0.05 * rng.standard_normal()) for bs in (4, 8, 16, 32, 64) for n in (32, 100, 300, 500)]
    b0, c0, k0 = S.fit_solo(pts)
    s = np.asarray(pts)
    X = np.stack([s[:, 0], np.ones(len(s)), s[:, 0] * s[:, 1]], axis=1)
    r = s[:, 2] - X @ np.array([b0, c0, k0])
    assert np.max(np.abs(X.T @ r)) < 1e-6 * np.max(np.abs(X.T @ s[:, 2]))
    # any perturbation of the coefficients increases the squared error
    base = float(r @ r)
    for d in itertools.product((-1, 0, 1), repeat=3):
        if d == (0, 0, 0):
            continue
        pert = np.array([b0, c0, k0]) * (1 + 1e-3 * np.array(d))
        rr = s[:, 2] - X @ pert
        assert float(rr @ rr) >= base


def test_eq2_recovers_the_bandwidth_sharing_model():
    # Sec. 5.2 theoretical analysis: slowdown = (f_infer + f_ft) / B with each demand proportional to its share
    cin, cft, B = 50.0, 30.0, 8.0      # demands large enough that every pair is in the contended regime
    pts = []
    for i, f in S.pairs(10):
        solo = 2.0 / (i / 10) ** 0.5
        pts.append((i / 10, f / 10, (cin * i / 10 + cft * f / 10) / B * solo, solo))
    b1, k1 = S.fit_colo(pts)
    assert abs(b1 - cin / B) < 1e-9 and abs(k1 - cft / B) < 1e-9
    assert abs(S.predict_colo((b1, k1), 0.4, 0.3, 3.0) - (0.4 * cin + 0.3 * cft) / B * 3.0) < 1e-9


def test_ten_levels_give_the_papers_45_plans():
    p = S.pairs(10)
    assert len(p) == 45 and len(set(p)) == 45
    assert all(1 <= i and 1 <= f and i + f <= 10 for i, f in p)
    assert (9, 1) in p and (1, 9) in p and (5, 5) in p and (9, 2) not in p


def _flat_solo(levels, lat_by_level):
    # Eq. 1 models with b0 = k0 = 0: latency depends on the ratio only
    return [(0.0, lat_by_level[i], 0.0) for i in range(levels)]


def test_pick_takes_the_plan_closest_below_the_target():
    solo = _flat_solo(10, [10.0, 6.0, 4.5, 3.8, 3.3, 3.0, 2.8, 2.6, 2.5, 2.4])
    colo = (10.0, 10.0)         # factor = i + f >= 2: contended everywhere
    # brute force by hand
    cands = [(i, f, (i + f) * solo[i - 1][1]) for i, f in S.pairs(10)]
    ok = [c for c in cands if c[2] <= 20.0]
    want = max(ok, key=lambda c: (c[2], c[1], -c[0]))
    got = S.pick(solo, colo, 8, 512, 20.0)
    assert got[:2] == want[:2] and abs(got[2] - want[2]) < 1e-12
    assert got[2] <= 20.0
    # nothing else that fits is closer to the target
    assert all(c[2] <= got[2] + 1e-12 for c in ok)


def test_pick_ties_go_to_the_larger_finetune_share():
    solo = _flat_solo(4, [4.0, 2.0, 4.0 / 3.0, 1.0])      # latency * ratio constant -> (i + f)/i * const
    colo = (4.0, 4.0)           # factor = i + f
    # pairs with the same predicted latency: (1,1): 2*4 = 8.0 ; (2,2): 4*2 = 8.0 -> f = 2 wins
    i, f, lat = S.pick(solo, colo, 1, 1, 8.0, n_levels=4)
    assert (i, f) == (2, 2) and abs(lat - 8.0) < 1e-12


def test_without_contention_the_colocated_latency_is_the_solo_latency():
    # factor 0.3*0.5 + 0.2*1.0 = 0.35 < 1: no contention (combined demand below the bandwidth) -> solo latency;
    # factor 0.8*0.5 + 0.2*4.0 = 1.2 -> 1.2 x solo
    assert S.predict_colo((0.5, 1.0), 0.3, 0.2, 3.0) == 3.0
    assert abs(S.predict_colo((0.5, 4.0), 0.8, 0.2, 3.0) - 3.6) < 1e-12
    # a neighbour never makes the predicted decode step faster, whatever the coefficients
    rng = np.random.default_rng(3)
    for _ in range(200):
        c = tuple(rng.uniform(0, 3, 2))
        i, f = S.pairs(10)[rng.integers(45)]
        assert S.predict_colo(c, i / 10, f / 10, 2.5) >= 2.5


def test_pick_pauses_finetune_when_no_plan_meets_the_target():
    solo = _flat_solo(10, [50.0] * 10)
    i, f, lat = S.pick(solo, (1.0, 1.0), 8, 512, 1.0)
    assert (i, f) == (10, 0) and lat == 50.0


# ---- runtime scheduling (Sec. 6.2): hand-worked traces on a model whose predictions can be done in the head ----
def _toy():
    """Solo latency = bs at every level (b0 = 1, c0 = k0 = 0); Eq. 2 with b1 = 0, k1 = 10: the slowdown factor is f
    (>= 1: contended), the co-located latency f * bs, independent of the inference share.  With a target of 40 the
    largest admissible finetune share is f = floor(40 / bs); ties (every i gives the same latency) go to the
    smallest inference share i = 1."""
    return [(1.0, 0.0, 0.0)] * 10, (0.0, 10.0)


def test_runtime_scheduler_follows_the_rules_of_sec_6_2():
    solo, colo = _toy()
    s = S.RuntimeScheduler(solo, colo, slo=40.0)
    assert s.step(8, 100, True) == (1, 5, 40.0, S.REPLAN)           # first phase: 8 f <= 40 -> f = 5
    assert s.step(8, 999, True) == (1, 5, 40.0, S.KEEP)             # still valid: both continue
    i, f, lat, act = s.step(10, 100, True)                         # 5 * 10 = 50 > 40: pause finetune, re-plan
    assert (i, f, act) == (1, 4, S.REPLAN) and abs(lat - 40.0) < 1e-12
    assert s.step(50, 100, True) == (10, 0, 50.0, S.PAUSED)        # 50 f <= 40 has no solution: inference alone
    assert s.step(50, 100, True) == (10, 0, 50.0, S.PAUSED)        # retried every phase
    assert s.step(8, 100, True) == (1, 5, 40.0, S.REPLAN)           # load fell: finetune resumes under a new plan
    assert s.step(8, 100, False) == (10, 0, 8.0, S.STARVED)        # no ready finetune work: all CUs to inference
    assert s.step(8, 100, True) == (1, 5, 40.0, S.REPLAN)           # work is back: redistribute


def test_runtime_scheduler_refresh_revisits_a_plan_that_stays_valid():
    solo, colo = _toy()
    s = S.RuntimeScheduler(solo, colo, slo=40.0, refresh_phases=3)
    assert s.step(20, 0, True)[:2] == (1, 2)                       # 20 f <= 40 -> f = 2
    assert s.step(5, 0, True) == (1, 2, 10.0, S.KEEP)               # valid, far below the target, age 1
    assert s.step(5, 0, True) == (1, 2, 10.0, S.KEEP)               # age 2
    assert s.step(5, 0, True) == (1, 8, 40.0, S.REPLAN)             # age 3: recomputed, 5 f <= 40 -> f = 8
    assert s.step(5, 0, True)[3] == S.KEEP and s.step(5, 0, True)[3] == S.KEEP
    assert s.step(5, 0, True) == (1, 8, 40.0, S.KEEP)               # age 3 again: same pair, nothing to do
    never = S.RuntimeScheduler(solo, colo, slo=40.0)
    never.step(20, 0, True)
    assert all(never.step(5, 0, True) == (1, 2, 10.0, S.KEEP) for _ in range(10))
