"""The library's host-side predictor and allocation choice against the oracle (CPU only: no GPU call is made).

Coefficients and predictions: both sides solve the same least-squares problems in double precision (QR in the
library, LAPACK in the oracle); they must agree to 1e-8 relative.  Chosen plans are integers and must be equal.
"""
import numpy as np
import pytest

from oracle import sched_oracle as S
from paper_2511_11729_amd import binding as hb


def synth_profile(seed, n_levels=10, noise=0.02, weak=False):
    """Latencies shaped like a decode step on a fraction of the chip: a weight-streaming floor that shrinks
    sublinearly with the compute-unit ratio plus per-sequence and per-token terms, with multiplicative noise."""
    rng = np.random.default_rng(seed)
    solo = {}
    for lv in range(1, n_levels + 1):
        r = lv / n_levels
        c0 = 0.09 / r ** 0.7 + 0.03
        b0 = 0.0015 / r ** 0.5
        k0 = 2.0e-6 / r ** 0.8
        solo[lv] = [(bs, n, (bs * b0 + c0 + bs * k0 * n) * (1 + noise * rng.standard_normal()))
                    for bs in (4, 16, 64) for n in (64, 128, 256, 512)]
    colo = []
    for i, f in S.pairs(n_levels):
        base = solo[i][5][2]
        # weak: slowdowns of a few percent, growing with the neighbour's share (partitions that barely contend)
        factor = 1.0 + 0.13 * f / n_levels if weak else 0.55 * i / n_levels + 0.9 + 0.8 * f / n_levels
        colo.append((i, f, base * factor * (1 + noise * rng.standard_normal()), base))
    return solo, colo


def build_both(seed, n_levels=10, noise=0.02, weak=False):
    solo, colo = synth_profile(seed, n_levels, noise, weak)
    p = hb.Predictor(n_levels)
    for lv, pts in solo.items():
        for bs, n, lat in pts:
            p.add_solo(lv, bs, n, lat)
    for i, f, lc, ls in colo:
        p.add_colo(i, f, lc, ls)
    p.fit()
    o_solo = [S.fit_solo(solo[lv]) for lv in range(1, n_levels + 1)]
    o_colo = S.fit_colo([(i / n_levels, f / n_levels, lc, ls) for i, f, lc, ls in colo])
    return p, o_solo, o_colo


@pytest.mark.parametrize("seed", [0, 1])
def test_calibration_scales_every_prediction_of_its_level(seed):
    p, o_solo, o_colo = build_both(seed)
    rng = np.random.default_rng(100 + seed)
    scales = rng.uniform(0.7, 1.8, 10)
    for lv in range(1, 11):
        p.set_scale(lv, float(scales[lv - 1]))
    cal = [S.calibrated(o_solo[lv], scales[lv]) for lv in range(10)]
    for lv in range(1, 11):
        assert np.allclose(p.solo_coef(lv), o_solo[lv - 1], rtol=1e-8, atol=1e-14)       # the fit itself is untouched
        want = S.predict_solo(cal[lv - 1], 24, 900)
        assert abs(p.solo(lv, 24, 900) - want) <= 1e-9 * abs(want)
    for i, f in S.pairs(10):
        want = S.predict_colo(o_colo, i / 10, f / 10, S.predict_solo(cal[i - 1], 8, 1153))
        assert abs(p.colo(i, f, 8, 1153) - want) <= 1e-8 * abs(want)
    for bs, n, slo in [(8, 512, 0.4), (42, 1024, 0.9), (24, 300, 0.25), (64, 2048, 3.0)]:
        wi, wf, wl_ = S.pick(cal, o_colo, bs, n, slo)
        gi, gf, gl = p.pick(bs, n, slo)
        assert (gi, gf) == (wi, wf) and abs(gl - wl_) <= 1e-8 * abs(wl_)
    ora = S.RuntimeScheduler(cal, o_colo, 0.6, 10, 8)
    sch = hb.Scheduler(p, 0.6, 8)
    for k in range(60):
        bs, n, ready = int(rng.integers(1, 80)), int(rng.integers(16, 2000)), bool(rng.random() > 0.1)
        assert sch.step(bs, n, ready)[:2] == ora.step(bs, n, ready)[:2]
    # one factor on every level is the same as dividing the target by it
    for lv in range(1, 11):
        p.set_scale(lv, 1.25)
    assert p.pick(24, 700, 0.5)[:2] == S.pick(o_solo, o_colo, 24, 700, 0.5 / 1.25)[:2]
    with pytest.raises(hb.HarliError):
        p.set_scale(11, 1.0)
    with pytest.raises(hb.HarliError):
        p.set_scale(3, 0.0)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("weak", [False, True])
def test_fits_and_predictions_match_the_oracle(seed, weak):
    p, o_solo, o_colo = build_both(seed, noise=0.004 if weak else 0.02, weak=weak)
    if weak:                                       # the regime where the floor decides which samples are fitted
        assert 0.7 < o_colo[0] < 1.3 and 0.9 < o_colo[1] < 1.5
    for lv in range(1, 11):
        got = p.solo_coef(lv)
        assert np.allclose(got, o_solo[lv - 1], rtol=1e-8, atol=1e-14), (lv, got, o_solo[lv - 1])
    assert np.allclose(p.colo_coef(), o_colo, rtol=1e-8)
    for lv, bs, n in [(1, 1, 0), (3, 8, 77), (10, 256, 4096), (7, 33, 1000)]:
        assert abs(p.solo(lv, bs, n) - S.predict_solo(o_solo[lv - 1], bs, n)) <= 1e-8 * abs(S.predict_solo(o_solo[lv - 1], bs, n))
    for i, f in S.pairs(10):
        want = S.predict_colo(o_colo, i / 10, f / 10, S.predict_solo(o_solo[i - 1], 8, 1153))
        assert abs(p.colo(i, f, 8, 1153) - want) <= 1e-8 * abs(want)


@pytest.mark.parametrize("weak", [False, True])
def test_eq2_as_printed_is_one_plain_fit_without_a_floor(weak):
    """Sec. 5.2.1 Eq. 2 as the paper prints it: with the floor switched off the library's fit is the ordinary
    least-squares solution over every sample and its predictions may fall below the solo latency."""
    n_levels = 10
    solo, colo = synth_profile(3, n_levels, 0.004 if weak else 0.02, weak)
    p, o_solo, o_floor = build_both(3, noise=0.004 if weak else 0.02, weak=weak)
    p.set_colo_floor(False)
    with pytest.raises(hb.HarliError):             # the co-located fit was discarded with the reading
        p.colo_coef()
    p.fit()
    samples = [(i / n_levels, f / n_levels, lc, ls) for i, f, lc, ls in colo]
    o_plain = S.fit_colo(samples, floor=False)
    X = np.array([[a * ls, b * ls] for a, b, _, ls in samples])
    y = np.array([lc for _, _, lc, _ in samples])
    normal = np.linalg.solve(X.T @ X, X.T @ y)     # the normal equations, written out
    assert np.allclose(o_plain, normal, rtol=1e-9)
    assert np.allclose(p.colo_coef(), o_plain, rtol=1e-8)
    below = 0
    for i, f in S.pairs(n_levels):
        base = S.predict_solo(o_solo[i - 1], 8, 1153)
        want = S.predict_colo(o_plain, i / 10, f / 10, base, floor=False)
        assert abs(want - (i / 10 * o_plain[0] + f / 10 * o_plain[1]) * base) <= 1e-12 * abs(want)
        assert abs(p.colo(i, f, 8, 1153) - want) <= 1e-8 * abs(want)
        below += want < base
    assert below > 0                               # e.g. 1/10 + 1/10: the printed form predicts a speed-up there
    p.set_colo_floor(True)
    p.fit()
    assert np.allclose(p.colo_coef(), o_floor, rtol=1e-8)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_chosen_plans_equal_the_oracles(seed):
    p, o_solo, o_colo = build_both(seed)
    rng = np.random.default_rng(100 + seed)
    n_paused = 0
    for _ in range(300):
        bs = int(rng.integers(1, 257))
        n = int(rng.integers(0, 4097))
        slo = float(rng.uniform(0.05, 3.0))
        gi, gf, gl = p.pick(bs, n, slo)
        wi, wf, wl_ = S.pick(o_solo, o_colo, bs, n, slo)
        assert (gi, gf) == (wi, wf), (bs, n, slo, (gi, gf, gl), (wi, wf, wl_))
        assert abs(gl - wl_) <= 1e-8 * abs(wl_)
        n_paused += gf == 0
        if gf:
            assert gl <= slo and gi + gf <= 10
    assert 0 < n_paused < 300          # both branches were exercised


def test_exact_data_gives_exact_coefficients():
    p = hb.Predictor(4)
    for lv in range(1, 5):
        for bs in (2, 8, 32):
            for n in (10, 100, 1000):
                p.add_solo(lv, bs, n, bs * 0.01 * lv + 0.5 / lv + bs * 1e-5 * n)
    p.fit()
    for lv in range(1, 5):
        assert np.allclose(p.solo_coef(lv), (0.01 * lv, 0.5 / lv, 1e-5), rtol=1e-9)


def test_errors():
    p = hb.Predictor(10)
    with pytest.raises(hb.HarliError):
        p.add_solo(0, 4, 100, 1.0)                # level out of range
    with pytest.raises(hb.HarliError):
        p.add_colo(6, 5, 1.0, 1.0)                # 6 + 5 > 10
    with pytest.raises(hb.HarliError):
        p.add_solo(1, 4, 100, float("nan"))
    p.add_solo(1, 4, 100, 1.0)
    p.add_solo(1, 4, 200, 1.1)
    with pytest.raises(hb.HarliError) as e:
        p.fit()                                   # two samples
    assert e.value.status == hb.HARLI_ERR_STATE
    p.add_solo(1, 4, 300, 1.2)
    with pytest.raises(hb.HarliError) as e:
        p.fit()                                   # one batch size only: rank deficient
    assert e.value.status == hb.HARLI_ERR_STATE
    with pytest.raises(hb.HarliError):
        p.pick(8, 100, 1.0)                       # nothing fitted
    with pytest.raises(hb.HarliError):
        hb.Predictor(1)


@pytest.mark.parametrize("seed,refresh", [(0, 0), (1, 4), (2, 1), (3, 16)])
def test_runtime_scheduler_matches_the_oracle_on_random_traces(seed, refresh):
    """400 decode phases of a random walk in batch size and sequence length with starvation episodes: the
    library's decisions (levels and action bit-exact, prediction to 1e-8) equal the oracle's at every phase."""
    p, o_solo, o_colo = build_both(seed)
    rng = np.random.default_rng(100 + seed)
    slo = float(rng.uniform(0.15, 0.6))
    lib_s = hb.Scheduler(p, slo, refresh)
    ora_s = S.RuntimeScheduler(o_solo, o_colo, slo, 10, refresh)
    bs, n = 8, 300
    seen = set()
    for _ in range(400):
        bs = int(np.clip(bs + rng.integers(-6, 7), 1, 96))
        n = int(np.clip(n + rng.integers(-200, 260), 0, 4096))
        ready = rng.random() > 0.1
        gi, gf, gl, ga = lib_s.step(bs, n, ready)
        wi, wf, wl_, wa = ora_s.step(bs, n, ready)
        assert (gi, gf, ga) == (wi, wf, wa), (bs, n, ready)
        assert abs(gl - wl_) <= 1e-8 * abs(wl_)
        seen.add(ga)
    assert {hb.SCHED_KEEP, hb.SCHED_REPLAN, hb.SCHED_STARVED} <= seen
    lib_s.close()


def test_runtime_scheduler_rejects_bad_arguments():
    p, _, _ = build_both(0)
    for slo, refresh in [(0.0, 0), (-1.0, 0), (1.0, -1)]:
        with pytest.raises(hb.HarliError) as e:
            hb.Scheduler(p, slo, refresh)
        assert e.value.status == hb.HARLI_ERR_INVALID
    unfitted = hb.Predictor(10)
    with pytest.raises(hb.HarliError) as e:
        hb.Scheduler(unfitted, 1.0, 0)
    assert e.value.status == hb.HARLI_ERR_STATE
    s = hb.Scheduler(p, 1.0, 0)
    for bs, n in [(0, 10), (4, -1)]:
        with pytest.raises(hb.HarliError):
            s.step(bs, n, True)


def test_run_time_feedback_equals_the_model_and_moves_the_predictions():
    p, o_solo, o_colo = build_both(0)
    rng = np.random.default_rng(77)
    c = S.Calibration(10)
    for k in range(300):
        lv = int(rng.integers(1, 11))
        pred, meas, wgt = float(rng.uniform(0.1, 40)), float(rng.uniform(0.05, 90)), float(rng.choice([0.15, 0.5, 1.0]))
        if k % 50 == 49:
            v = float(rng.uniform(0.7, 1.5))
            c.set(lv, v)
            p.set_scale(lv, v)
        c.observe(lv, pred, meas, wgt)
        p.observe(lv, pred, meas, wgt)
        got = [p.get_scale(l) for l in range(1, 11)]
        assert np.allclose(got, c.scale, rtol=1e-12, atol=0)
    for lv in range(1, 11):                         # and the factor is what every prediction of the level carries
        want = S.predict_solo(S.calibrated(o_solo[lv - 1], c.scale[lv - 1]), 24, 900)
        assert abs(p.solo(lv, 24, 900) - want) <= 1e-9 * abs(want)
    for bad in [(0, 1.0, 1.0, 0.5), (11, 1.0, 1.0, 0.5), (1, 0.0, 1.0, 0.5), (1, 1.0, -1.0, 0.5), (1, 1.0, 1.0, 0.0),
                (1, 1.0, 1.0, 1.5), (1, float("nan"), 1.0, 0.5), (1, 1.0, float("inf"), 0.5)]:
        with pytest.raises(hb.HarliError) as e:
            p.observe(*bad)
        assert e.value.status == hb.HARLI_ERR_INVALID


# ---- Eq. 1 per kernel family (batch split) -------------------------------------------------------------------------
def two_family_samples(rng, lv, noise=0.0, upper_batches=(40, 64, 160), knee=33):
    """Step times that are linear in the batch size on either side of `knee` with different slopes (the shape of a
    decode step that switches kernel families there)."""
    r = lv / 10.0
    lo = (0.0016 / r ** 0.5, 0.09 / r ** 0.7 + 0.03, 2.0e-6 / r ** 0.8)
    hi = (0.0007 / r ** 0.5, 0.13 / r ** 0.7 + 0.05, 1.6e-6 / r ** 0.8)
    pts = []
    for bs in (4, 16) + tuple(upper_batches):
        b0, c0, k0 = hi if bs >= knee else lo
        for n in (64, 128, 256, 512):
            pts.append((bs, n, (bs * b0 + c0 + bs * k0 * n) * (1 + noise * rng.standard_normal())))
    return pts, lo, hi


def test_oracle_split_fit_recovers_both_lines_exactly_from_noiseless_samples():
    """Pin of the oracle's own split fit: samples generated from two known lines give those lines back, one plain line
    through all of them does not, and a family with a single batch size borrows the other family's line."""
    rng = np.random.default_rng(0)
    pts, lo, hi = two_family_samples(rng, 5)
    c = S.fit_solo_split(pts, 33)
    assert np.allclose(c.lo, lo, rtol=1e-9) and np.allclose(c.hi, hi, rtol=1e-9)
    for bs, n, lat in pts:
        assert abs(S.predict_solo(c, bs, n) - lat) <= 1e-9 * lat
    one = S.fit_solo(pts)
    assert max(abs(S.predict_solo(one, bs, n) - lat) / lat for bs, n, lat in pts) > 0.05
    # the upper family measured at one batch size only: its line is not determined
    pts1, lo1, _ = two_family_samples(rng, 5, upper_batches=(64,))
    c1 = S.fit_solo_split(pts1, 33)
    assert np.allclose(c1.lo, lo1, rtol=1e-9) and c1.hi == c1.lo
    # a split below every sample: the lower family is empty and borrows the upper line, which is the plain fit
    c2 = S.fit_solo_split(pts, 2)
    assert np.allclose(c2.lo, one, rtol=1e-9) and np.allclose(c2.hi, one, rtol=1e-9)
    with pytest.raises(ValueError):
        S.fit_solo_split(pts[:2], 33)


@pytest.mark.parametrize("seed", [0, 1])
def test_batch_split_in_the_library_matches_the_oracle(seed):
    rng = np.random.default_rng(40 + seed)
    p = hb.Predictor(10)
    o = []
    samples = {}
    for lv in range(1, 11):
        pts, _, _ = two_family_samples(rng, lv, noise=0.01, upper_batches=(64,) if lv == 4 else (40, 64, 160))
        samples[lv] = pts
        for bs, n, lat in pts:
            p.add_solo(lv, bs, n, lat)
    colo = [(i, f, 1.0 + 0.1 * f, 1.0) for i, f in S.pairs(10)]
    for i, f, lc, ls in colo:
        p.add_colo(i, f, lc, ls)
    p.fit()
    plain = [S.fit_solo(samples[lv]) for lv in range(1, 11)]
    for lv in range(1, 11):                          # no split: one line, and the upper coefficients are the same line
        assert np.allclose(p.solo_coef(lv), plain[lv - 1], rtol=1e-8, atol=1e-14)
        assert p.solo_coef_upper(lv) == p.solo_coef(lv)
    p.set_batch_split(33)
    with pytest.raises(hb.HarliError):               # the lines of the other reading are gone
        p.solo_coef(1)
    p.fit()
    o = [S.fit_solo_split(samples[lv], 33) for lv in range(1, 11)]
    o_colo = S.fit_colo([(i / 10, f / 10, lc, ls) for i, f, lc, ls in colo])
    for lv in range(1, 11):
        assert np.allclose(p.solo_coef(lv), o[lv - 1].lo, rtol=1e-8, atol=1e-14)
        assert np.allclose(p.solo_coef_upper(lv), o[lv - 1].hi, rtol=1e-8, atol=1e-14)
        for bs, n in [(1, 0), (32, 500), (33, 500), (200, 1500)]:
            want = S.predict_solo(o[lv - 1], bs, n)
            assert abs(p.solo(lv, bs, n) - want) <= 1e-8 * abs(want)
    assert p.solo_coef_upper(4) == p.solo_coef(4)    # level 4 saw one batch size above the split
    # the split line predicts the upper family better than the single line did
    lv = 7
    err_split = np.mean([abs(S.predict_solo(o[lv - 1], bs, n) - lat) / lat for bs, n, lat in samples[lv]])
    err_plain = np.mean([abs(S.predict_solo(plain[lv - 1], bs, n) - lat) / lat for bs, n, lat in samples[lv]])
    assert err_split < 0.02 < err_plain
    # allocation choices and the runtime scheduler follow the split predictions
    for bs, n, slo in [(8, 512, 0.4), (42, 1024, 0.9), (150, 300, 0.6), (64, 2048, 3.0)]:
        wi, wf, wl_ = S.pick(o, o_colo, bs, n, slo)
        gi, gf, gl = p.pick(bs, n, slo)
        assert (gi, gf) == (wi, wf) and abs(gl - wl_) <= 1e-8 * abs(wl_)
    ora = S.RuntimeScheduler(o, o_colo, 0.6, 10, 8)
    sch = hb.Scheduler(p, 0.6, 8)
    for k in range(80):
        bs, n, ready = int(rng.integers(1, 200)), int(rng.integers(16, 2000)), bool(rng.random() > 0.1)
        assert sch.step(bs, n, ready)[:2] == ora.step(bs, n, ready)[:2]
    p.set_batch_split(0)
    p.fit()
    assert np.allclose(p.solo_coef(7), plain[6], rtol=1e-8, atol=1e-14)
    with pytest.raises(hb.HarliError):
        p.set_batch_split(-1)


def test_tiled_min_batch_is_reported():
    assert hb.decode_tiled_min_batch() == 33
