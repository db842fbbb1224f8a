"""CPU oracle of the latency predictor and the allocation choice (Harli Sec. 5 and Sec. 6.2).

TEST INFRASTRUCTURE ONLY: plain NumPy float64, written from the paper's equations; the product path never
imports it.  It is the definition the library's host-side predictor (`harli_pred_*`, `harli_sched_pick`) is
compared with.

* Eq. 1 (solo decode latency, one model per compute-unit ratio):
      latency = bs*b0 + c0 + bs*k0*seqlen
  fitted by ordinary least squares over profiled (bs, seqlen, latency) samples.
  Addition to the paper (SplitCoef, fit_solo_split): one such line per kernel family of the decode step under test,
  samples and predictions below a batch threshold using one set of coefficients and those from it on another;
  pinned by samples drawn from two known lines, which the split fit gives back and a single line cannot.
* Eq. 2 (co-located decode latency):
      latency_colo = (SM_infer*b1 + SM_ft*k1) * latency_solo(SM_infer)
  fitted by ordinary least squares of latency_colo on the two regressors SM_infer*latency_solo and
  SM_ft*latency_solo (the paper says only that b1, k1 come from profiling; this is the reading taken).
  Prediction floors the factor at 1: the theoretical analysis of Sec. 5.2 derives it as
  (f_infer + f_ft) / B under contention, f_infer + f_ft > B, where it is at least 1; with less combined demand
  than bandwidth the tasks do not slow each other and the co-located latency is the solo latency (a factor
  below 1 would predict that a neighbour makes decode faster).  The fit follows the same reading: a sample whose
  fitted factor is below 1 is predicted by the floor, whatever b1 and k1 are, so it says nothing about them;
  after the first least-squares pass over all samples the pass is repeated over the samples whose current
  factor is at least 1, until that set no longer changes (a stationary point of the squared error of the
  floored prediction).  With every sample in the contended regime this is the plain least-squares fit.
* Allocation (Sec. 5.2 "Perceive the Finetune Performance", Sec. 6.2): with ratios in steps of 1/n_levels the
  candidate plans are the pairs (SM_infer, SM_ft) with SM_infer + SM_ft <= 1, both at least one step (45 pairs
  for ten levels).  The plan chosen is the one whose predicted co-located latency is closest to the QoS target
  without exceeding it; ties go to the larger finetune share, then to the smaller inference share.  When no
  pair meets the target the finetune task is paused and inference gets every compute unit.
"""
from __future__ import annotations

import numpy as np


def fit_solo(samples):
    """samples: iterable of (bs, seqlen, latency).  Returns (b0, c0, k0) of Eq. 1."""
    s = np.asarray(list(samples), np.float64)
    X = np.stack([s[:, 0], np.ones(len(s)), s[:, 0] * s[:, 1]], axis=1)
    beta, *_ = np.linalg.lstsq(X, s[:, 2], rcond=None)
    return tuple(float(b) for b in beta)


class SplitCoef:
    """Eq. 1 per kernel family (an addition to the paper's predictor, which has one line per compute-unit level):
    `lo` = (b0, c0, k0) for batches below `bs_split`, `hi` for batches from `bs_split` on.  The decode step under
    test runs two kernel families whose step times are linear in the batch size with different slopes."""

    def __init__(self, bs_split, lo, hi):
        self.bs_split, self.lo, self.hi = int(bs_split), tuple(lo), tuple(hi)


def _determined(s):
    """Do the samples fix a line of Eq. 1?  Three of them with a design matrix of full rank."""
    if len(s) < 3:
        return False
    s = np.asarray(s, np.float64)
    X = np.stack([s[:, 0], np.ones(len(s)), s[:, 0] * s[:, 1]], axis=1)
    return int(np.linalg.matrix_rank(X)) == 3


def fit_solo_split(samples, bs_split):
    """One least-squares fit of Eq. 1 per family; a family its samples do not determine takes the other's line."""
    samples = list(samples)
    lo = [t for t in samples if t[0] < bs_split]
    hi = [t for t in samples if t[0] >= bs_split]
    ok_lo, ok_hi = _determined(lo), _determined(hi)
    if not ok_lo and not ok_hi:
        raise ValueError("the samples determine neither line")
    c_lo = fit_solo(lo) if ok_lo else None
    c_hi = fit_solo(hi) if ok_hi else None
    return SplitCoef(bs_split, c_lo if ok_lo else c_hi, c_hi if ok_hi else c_lo)


def predict_solo(coef, bs, seqlen):
    if isinstance(coef, SplitCoef):
        coef = coef.hi if bs >= coef.bs_split else coef.lo
    b0, c0, k0 = coef
    return bs * b0 + c0 + bs * k0 * seqlen


def calibrated(coef, scale):
    """Eq. 1 coefficients whose prediction is `scale` times that of `coef` (the library's per-level calibration
    factor, an addition to the paper's predictor: measured / predicted, folded back in at run time)."""
    if isinstance(coef, SplitCoef):
        return SplitCoef(coef.bs_split, calibrated(coef.lo, scale), calibrated(coef.hi, scale))
    return tuple(scale * c for c in coef)


SCALE_MIN, SCALE_MAX = 0.6, 2.5


class Calibration:
    """Run-time feedback into the per-level calibration factors (an addition to the paper's scheduler, which plans with
    the fitted predictor alone, Sec. 6.2).  One finished decode step at a level gives r = measured / predicted (the
    prediction without the factor), clipped to [SCALE_MIN, SCALE_MAX]: the first step seen at a level sets its factor
    to r, later ones move it by weight * (r - factor); levels with no step seen yet take the new factor of the level
    just measured.  Setting a factor by hand makes the level unseen again."""

    def __init__(self, n_levels: int):
        self.scale = [1.0] * n_levels          # index level - 1
        self.seen = [False] * n_levels

    def set(self, level: int, scale: float):
        self.scale[level - 1] = float(scale)
        self.seen[level - 1] = False

    def observe(self, level: int, predicted_ms: float, measured_ms: float, weight: float):
        r = min(SCALE_MAX, max(SCALE_MIN, measured_ms / predicted_ms))
        i = level - 1
        self.scale[i] = self.scale[i] + weight * (r - self.scale[i]) if self.seen[i] else r
        self.seen[i] = True
        for j in range(len(self.scale)):
            if not self.seen[j]:
                self.scale[j] = self.scale[i]


COLO_FIT_ROUNDS = 32


def fit_colo(samples, floor=True):
    """samples: iterable of (sm_infer, sm_ft, latency_colo, latency_solo_at_sm_infer).  Returns (b1, k1) of Eq. 2.
    floor=False is Eq. 2 as printed: one least-squares fit over every sample."""
    s = np.asarray(list(samples), np.float64)
    X = np.stack([s[:, 0] * s[:, 3], s[:, 1] * s[:, 3]], axis=1)
    beta, *_ = np.linalg.lstsq(X, s[:, 2], rcond=None)
    active = np.ones(len(s), bool)
    for _ in range(COLO_FIT_ROUNDS if floor else 0):
        now = s[:, 0] * beta[0] + s[:, 1] * beta[1] >= 1.0      # samples the floor does not cover
        if (now == active).all() or now.sum() < 2 or np.linalg.matrix_rank(X[now]) < 2:
            break
        active = now
        beta, *_ = np.linalg.lstsq(X[active], s[active, 2], rcond=None)
    return float(beta[0]), float(beta[1])


def predict_colo(colo_coef, sm_infer, sm_ft, latency_solo, floor=True):
    """Eq. 2 with the slowdown factor floored at 1 (see the module header); floor=False: Eq. 2 as printed."""
    b1, k1 = colo_coef
    factor = sm_infer * b1 + sm_ft * k1
    return (max(1.0, factor) if floor else factor) * latency_solo


def pairs(n_levels=10):
    """Index pairs (i, f), 1-based numbers of steps, with i + f <= n_levels."""
    return [(i, f) for i in range(1, n_levels) for f in range(1, n_levels - i + 1)]


def pick(solo_coefs, colo_coef, bs, seqlen, slo, n_levels=10):
    """solo_coefs[i-1] = Eq. 1 coefficients at ratio i/n_levels.  Returns (i, f, predicted latency); f = 0 means
    the finetune task is paused and inference runs alone on all compute units (i = n_levels)."""
    best = None
    for i, f in pairs(n_levels):
        lat = predict_colo(colo_coef, i / n_levels, f / n_levels, predict_solo(solo_coefs[i - 1], bs, seqlen))
        if lat > slo:
            continue
        key = (lat, f, -i)
        if best is None or key > best[0]:
            best = (key, (i, f, lat))
    if best is None:
        return n_levels, 0, predict_solo(solo_coefs[n_levels - 1], bs, seqlen)
    return best[1]


KEEP, REPLAN, PAUSED, STARVED = 0, 1, 2, 3


class RuntimeScheduler:
    """Per-decode-phase allocation decisions (Sec. 6.2 "Runtime Scheduling").

    Called once at the beginning of every decode phase with the batch size, the sequence length and whether the
    finetune task has ready work.  Returns (infer_level, ft_level, predicted latency, action):

    * the finetune task has no ready work (it waits for data): inference takes every compute unit for this phase
      (STARVED); the plan is recomputed when the finetune task is ready again;
    * no plan in force (first phase, after a starved or paused phase): the closest-below-target plan is chosen
      (REPLAN), or, when no plan meets the target, the finetune task stays paused and inference runs alone on the
      whole chip (PAUSED);
    * a plan is in force: its co-located latency is predicted for the new (bs, seqlen); above the target, the
      finetune task is paused and a new plan is computed (REPLAN, or PAUSED when none qualifies); otherwise both
      tasks continue (KEEP).
    * Reading taken where the paper is silent: a plan that stays valid while the load falls would never be
      revisited by the rules above, yet Sec. 8.6 reports adjustments about every 100 ms.  After `refresh_phases`
      consecutive phases under one plan (0 = never) the choice is recomputed; REPLAN if it differs, KEEP if not.
    """

    def __init__(self, solo_coefs, colo_coef, slo, n_levels=10, refresh_phases=0):
        self.solo_coefs, self.colo_coef, self.slo, self.n, self.refresh = solo_coefs, colo_coef, slo, n_levels, refresh_phases
        self.cur = None
        self.age = 0

    def _solo_full(self, bs, seqlen):
        return predict_solo(self.solo_coefs[self.n - 1], bs, seqlen)

    def _replan(self, bs, seqlen):
        i, f, lat = pick(self.solo_coefs, self.colo_coef, bs, seqlen, self.slo, self.n)
        self.age = 0
        if f == 0:
            self.cur = None
            return i, f, lat, PAUSED
        self.cur = (i, f)
        return i, f, lat, REPLAN

    def step(self, bs, seqlen, ft_ready):
        if not ft_ready:
            self.cur = None
            self.age = 0
            return self.n, 0, self._solo_full(bs, seqlen), STARVED
        if self.cur is None:
            return self._replan(bs, seqlen)
        i, f = self.cur
        lat = predict_colo(self.colo_coef, i / self.n, f / self.n, predict_solo(self.solo_coefs[i - 1], bs, seqlen))
        if lat > self.slo:
            return self._replan(bs, seqlen)
        self.age += 1
        if self.refresh > 0 and self.age >= self.refresh:
            old = self.cur
            r = self._replan(bs, seqlen)
            if r[3] == REPLAN and self.cur == old:
                return r[0], r[1], r[2], KEEP
            return r
        return i, f, lat, KEEP
