"""Profiling and scheduling of the co-location on compute-unit partitions (Harli Sec. 5, Sec. 6.2).

`profile(hz)` measures one layer's decode latency on the device at ten compute-unit levels (streams restricted to
a contiguous range of compute units, an equal share of every XCD), fits Eq. 1 per level and Eq. 2 over the 45
disjoint (inference, finetune) partitions with the library's predictor, and reports the prediction errors on
held-out points.  `run_colocated(hz, ...)` runs decode and finetune side by side on given streams and returns
throughput and latency statistics.  Host orchestration only: timing uses HIP events on the streams involved.
"""
from __future__ import annotations

import gc
import threading
import time

import numpy as np
import torch

from . import binding as hb

N_LEVELS = 10
PROFILE_BATCHES = (4, 16, 32, 40, 64)      # representative batch sizes (Sec. 5.1), on either side of the library's switch of kernel families
PROFILE_SEQLENS = (64, 128, 256, 512)
HELDOUT = ((8, 96), (8, 384), (24, 192), (24, 448), (48, 320))


class CuStreams:
    """Streams restricted to compute-unit ranges, wrapped for torch; destroyed on close()."""

    def __init__(self):
        self.n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        self._raw = []
        self._big = self._small = None
        self.shared_pipe = []                      # partitions whose two streams ended up on one pipe (see pairs)
        self.unrestricted = None                   # after pairs(): an ordinary stream that shares a pipe with no inference stream

    def make(self, first: int, count: int):
        raw = hb.cu_stream_create(first, count)
        self._raw.append(raw)
        st = torch.cuda.ExternalStream(raw)
        if self._small is None:
            self._small = torch.zeros(64, dtype=torch.float32, device="cuda:0")
        with torch.cuda.stream(st):                # the hardware queue behind a stream is set up at its first use:
            self._small.add_(1.0)                  # do that here, not inside somebody's timed region
        st.synchronize()
        return st

    def low(self, level: int):
        """The first level/N_LEVELS of the compute units (inference side)."""
        return self.make(0, max(1, self.n_cu * level // N_LEVELS))

    def high(self, level: int):
        """The last level/N_LEVELS of the compute units (finetune side): disjoint from low(i) when i + level <= N."""
        c = max(1, self.n_cu * level // N_LEVELS)
        return self.make(self.n_cu - c, c)

    def _drop(self, streams):
        """Destroys streams made by make() (idle ones: candidates that were only probed)."""
        torch.cuda.synchronize()
        for st in streams:
            raw = st.cuda_stream
            if raw in self._raw:
                self._raw.remove(raw)
                hb.cu_stream_destroy(raw)

    def _conflict(self, a, b):
        """True when work on stream `a` queues behind work on stream `b` although their compute units are disjoint:
        the two sit on the same dispatch pipe.  A long element-wise kernel goes to `b`, a tiny one to `a` right after;
        on one pipe the tiny one ends only when the long one is nearly through.  Both ends are timed from the start
        of the long kernel (an event on `a` itself would queue behind the long kernel as well); asked twice, so that
        a one-off stall of the device is not taken for queueing."""
        if self._big is None:
            self._big = torch.zeros(96 << 20, dtype=torch.float32, device="cuda:0")
        for _ in range(2):
            torch.cuda.synchronize()
            eb0, eb1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ea1 = torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(b):
                eb0.record()
                self._big.add_(1.0)
                eb1.record()
            with torch.cuda.stream(a):
                self._small.add_(1.0)
                ea1.record()
            a.synchronize()
            b.synchronize()
            if eb0.elapsed_time(ea1) <= 0.5 * eb0.elapsed_time(eb1):
                return False
        return True

    def conflicts(self, low, high):
        """The (i, f) with i + f <= N whose streams low[i] and high[f] share a dispatch pipe."""
        return [(i, f) for i in sorted(low) for f in sorted(high) if i + f <= N_LEVELS and self._conflict(high[f], low[i])]

    def pairs(self, log=lambda *a: None):
        """(low, high): for every level an inference stream on the first level/N of the compute units and a finetune
        stream on the last level/N, such that no inference stream shares a dispatch pipe with a finetune stream it can
        run beside.  Two streams on one pipe dispatch their kernels one after the other: measured, a decode stream
        sharing a pipe with the finetune stream sees about twice the latency of one that does not.  Which pipe (of
        four) a stream's hardware queue sits on follows from its position among ALL hardware queues of the process,
        and the positions are dealt again whenever a queue is created or destroyed; so all eighteen restricted
        streams are created first, in an alternating order that usually keeps the two sides apart, and the result is
        then checked by measurement (`conflicts`); on a conflict everything is destroyed and another arrangement
        tried.  Level N (every compute unit; the finetune task is paused then, but units already in flight finish on
        their partition) is an ordinary stream, chosen among four so that it shares a pipe with no finetune stream.
        Call this after every other stream of the process exists AND has run something (the hardware queue behind
        an ordinary stream comes into being at its first use), and create none while the result is in use.
        Only the streams returned (and up to three idle spacers) stay alive: every restricted stream is a hardware
        queue of its own, ordinary streams share up to four, and measured, a process with 24 queues or more
        oversubscribes the queue slots of the device: every stream of the process then sees stalls of 10-30 ms."""
        if self._small is None:
            self._small = torch.zeros(64, dtype=torch.float32, device="cuda:0")
        cands = [torch.cuda.Stream() for _ in range(4)]    # level N (every compute unit) is an ordinary stream: one of
        for c in cands:                                    # these, chosen below; all used once now, so that the
            with torch.cuda.stream(c):                     # hardware queues behind them exist before the positions
                self._small.add_(1.0)                      # are measured
        torch.cuda.synchronize()

        def arrange(spacers):
            made = [self.low(1) for _ in range(spacers)]
            low, high = {}, {}
            for lv in range(1, N_LEVELS):
                low[lv] = self.low(lv)
                high[lv] = self.high(lv)
            # the full-chip stream runs beside finetune units still in flight on their partition after a pause
            clean = [c for c in cands if not any(self._conflict(c, high[f]) for f in high)]
            low[N_LEVELS] = clean[0] if clean else cands[0]
            # an ordinary stream (every compute unit) for a finetune task that is not restricted: on no inference pipe
            free = [c for c in cands if c is not low[N_LEVELS] and not any(self._conflict(c, low[i]) for i in range(1, N_LEVELS))]
            self.unrestricted = free[0] if free else None
            bad = self.conflicts(low, high) + ([] if clean else [(N_LEVELS, 0)])
            return made, low, high, bad

        best = None
        for spacers in (0, 1, 2, 3):
            made, low, high, bad = arrange(spacers)
            log("[streams] %d spacer(s): %d of 45 partitions share a pipe %s" % (spacers, len(bad), bad[:6]))
            if not bad:
                self.shared_pipe = []
                return low, high
            if best is None or len(bad) < best[0]:
                best = (len(bad), spacers)
            self._drop(made + [low[lv] for lv in range(1, N_LEVELS)] + list(high.values()))
        made, low, high, self.shared_pipe = arrange(best[1])   # none was clean: the arrangement with the fewest conflicts
        return low, high

    def close(self):
        """Destroys the streams.  Call it once nothing refers to them any more: no task still issues work on them and
        the events recorded on them have been let go (collected here before the streams go)."""
        gc.collect()
        torch.cuda.synchronize()
        for r in self._raw:
            hb.cu_stream_destroy(r)
        self._raw = []


def time_decode(hz, stream, batch, kv_len_dev, max_kv, steps):
    """Median latency in ms of `steps` decode steps issued back to back on `stream` (completion to completion;
    the median keeps one-off stalls of the host threads out of the profile)."""
    for _ in range(2):
        hz.decode_launch(stream, batch, kv_len_dev, max_kv)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record(stream)
    for k in range(steps):
        hz.decode_launch(stream, batch, kv_len_dev, max_kv)
        ev[k + 1].record(stream)
    stream.synchronize()
    return float(np.median([ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]))


class FinetuneLoop:
    """Keeps finetune units enqueued on a stream from a host thread until stopped (the neighbour in profiling).
    An exception in the thread ends it and is raised again in the thread that waits for it."""

    def __init__(self, hz, stream):
        self.hz, self.stream = hz, stream
        self.stop_flag = threading.Event()
        self.units = 0
        self.error = None
        self.th = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        try:
            torch.cuda.set_device(0)
            while not self.stop_flag.is_set():
                self.hz.finetune_unit(self.stream)
                self.units += 1
        except BaseException as e:                 # noqa: BLE001 -- handed to the waiting thread
            self.error = e

    def __enter__(self):
        self.th.start()
        while self.units < 2:
            if self.error is not None:
                self.th.join()
                raise RuntimeError("the finetune thread failed") from self.error
            time.sleep(1e-3)
        return self

    def __exit__(self, *a):
        self.stop_flag.set()
        self.th.join()
        self.stream.synchronize()
        if self.error is not None and a[0] is None:
            raise RuntimeError("the finetune thread failed") from self.error


def _quiesce(hz):
    """Before restricted streams are destroyed the harness lets go of the events it recorded on them."""
    drain = getattr(hz, "drain", None)
    if drain is not None:
        drain()


def profile(hz, steps=12, log=lambda *a: None, batches=None, seqlens=None, heldout=None):
    """Returns (predictor, report).  hz must have decode capacity for the largest profiled batch and length (default:
    the paper's grid, batch 4 / 16 / 64 at up to 512 cached tokens, plus batch 40); `decode_launch(stream, None, None,
    None)` runs the workload's own batch, the base of the co-located samples.  Eq. 1 is fitted per kernel family of the
    decode step (harli_pred_set_batch_split at the batch where the library switches to tiled GEMMs) when the grid has
    two batch sizes on either side; the report carries the error of the single line (Eq. 1 as printed) beside it."""
    PROFILE_BATCHES_, PROFILE_SEQLENS_, HELDOUT_ = batches or PROFILE_BATCHES, seqlens or PROFILE_SEQLENS, heldout or HELDOUT
    cs = CuStreams()
    pred = hb.Predictor(N_LEVELS)
    dev = hz.x_dev.device

    def lens(bs, n):
        return torch.full((bs,), n, dtype=torch.int32, device=dev)

    low, high = cs.pairs()
    solo_meas = {}
    t0 = time.perf_counter()
    for lv in range(1, N_LEVELS + 1):
        for bs in PROFILE_BATCHES_:
            for n in PROFILE_SEQLENS_:
                ms = time_decode(hz, low[lv], bs, lens(bs, n), n + 1, steps)
                pred.add_solo(lv, bs, n, ms)
                solo_meas[(lv, bs, n)] = ms
    held = {}
    for lv in range(1, N_LEVELS + 1):
        for bs, n in HELDOUT_:
            held[(lv, bs, n)] = time_decode(hz, low[lv], bs, lens(bs, n), n + 1, steps)
    # the workload's own batch (mixed lengths) solo at every level: the base of the co-located samples
    base = {lv: time_decode(hz, low[lv], None, None, None, steps) for lv in range(1, N_LEVELS + 1)}
    log("[sched] solo profile: %d + %d points in %.1f s" % (len(solo_meas), len(held), time.perf_counter() - t0))
    t0 = time.perf_counter()
    colo_meas = {}
    for f in range(1, N_LEVELS):
        with FinetuneLoop(hz, high[f]):
            for i in range(1, N_LEVELS - f + 1):
                colo_meas[(i, f)] = time_decode(hz, low[i], None, None, None, steps)
        for i in range(1, N_LEVELS - f + 1):
            pred.add_colo(i, f, colo_meas[(i, f)], base[i])
    log("[sched] co-located profile: %d partitions in %.1f s" % (len(colo_meas), time.perf_counter() - t0))
    # Eq. 2 as printed first (one least-squares fit, no floor), for the paper's accuracy figure; then the floored
    # reading the scheduler runs on
    pred.set_colo_floor(False)
    pred.fit()
    b1p, k1p = pred.colo_coef()
    err_printed = [abs((i / N_LEVELS * b1p + f / N_LEVELS * k1p) * base[i] - ms) / ms for (i, f), ms in colo_meas.items()]
    pred.set_colo_floor(True)
    pred.fit()
    # Eq. 1 as printed (one line per level) for the paper's accuracy figure; then one line per kernel family
    err_fit1 = [abs(pred.solo(lv, bs, n) - ms) / ms for (lv, bs, n), ms in solo_meas.items()]
    err_held1 = [abs(pred.solo(lv, bs, n) - ms) / ms for (lv, bs, n), ms in held.items()]
    split = hb.decode_tiled_min_batch()
    use_split = len([b for b in PROFILE_BATCHES_ if b >= split]) >= 2 and len([b for b in PROFILE_BATCHES_ if b < split]) >= 2
    if use_split:
        pred.set_batch_split(split)
        pred.fit()
    err_fit = [abs(pred.solo(lv, bs, n) - ms) / ms for (lv, bs, n), ms in solo_meas.items()]
    err_held = [abs(pred.solo(lv, bs, n) - ms) / ms for (lv, bs, n), ms in held.items()]
    b1, k1 = pred.colo_coef()
    err_colo = [abs(max(1.0, i / N_LEVELS * b1 + f / N_LEVELS * k1) * base[i] - ms) / ms for (i, f), ms in colo_meas.items()]
    report = {
        "levels": N_LEVELS, "compute_units": cs.n_cu,
        "eq1_mean_abs_err_fitted_points": float(np.mean(err_fit)), "eq1_mean_abs_err_heldout": float(np.mean(err_held)),
        "eq1_max_abs_err_heldout": float(np.max(err_held)),
        "eq1_batch_split": split if use_split else 0,
        "eq1_as_printed_mean_abs_err_fitted_points": float(np.mean(err_fit1)),
        "eq1_as_printed_mean_abs_err_heldout": float(np.mean(err_held1)),
        "eq1_as_printed_max_abs_err_heldout": float(np.max(err_held1)),
        "eq1_coef_full_chip_b0_c0_k0_ms": list(pred.solo_coef(N_LEVELS)),
        "eq2_b1_k1": [b1, k1], "eq2_mean_abs_err": float(np.mean(err_colo)), "eq2_max_abs_err": float(np.max(err_colo)),
        "eq2_as_printed_b1_k1": [b1p, k1p], "eq2_as_printed_mean_abs_err": float(np.mean(err_printed)),
        "eq2_as_printed_max_abs_err": float(np.max(err_printed)),
        "solo_ms_by_level_workload_batch": [base[lv] for lv in range(1, N_LEVELS + 1)],
        "colo_ms": {"%d+%d" % k: v for k, v in sorted(colo_meas.items())},
    }
    _quiesce(hz)
    cs.close()
    return pred, report


def run_colocated(hz, sD, sF, decode_once, K, W, pace_ms=None, finetune=True):
    """K timed finetune units on sF with decode on sD beside them (decode_once() issues one step on sD).
    pace_ms None: decode steps back to back; otherwise one step every pace_ms.  With finetune False only decode
    runs, for K * 3 ms.  Returns tokens/s, ms per unit, decode completion-to-completion intervals and step
    latencies (ms) inside the timed window."""
    stop = threading.Event()
    started = threading.Event()
    dec_start, dec_end = [], []

    def decode_thread():
        torch.cuda.set_device(0)
        i = 0
        t_next = time.perf_counter()
        while not stop.is_set():
            if pace_ms is not None:
                while True:
                    now = time.perf_counter()
                    if now >= t_next or stop.is_set():
                        break
                    time.sleep(min(2e-4, t_next - now))
                t_next = max(t_next + pace_ms * 1e-3, time.perf_counter() - 5 * pace_ms * 1e-3)
            if i >= 256:
                dec_end[i - 256].synchronize()         # bound the run-ahead of the host thread
            e0 = torch.cuda.Event(enable_timing=True)
            e0.record(sD)
            decode_once()
            e1 = torch.cuda.Event(enable_timing=True)
            e1.record(sD)
            dec_start.append(e0)
            dec_end.append(e1)
            i += 1
            if i == 8:
                started.set()

    th = threading.Thread(target=decode_thread, daemon=True)
    th.start()
    started.wait()
    if finetune:
        for _ in range(W):
            hz.finetune_unit(sF)
        sF.synchronize()
    torch.cuda.synchronize()
    i0 = len(dec_end)
    t0 = time.perf_counter()
    if finetune:
        for _ in range(K):
            hz.finetune_unit(sF)
        sF.synchronize()
    else:
        time.sleep(K * 3e-3)
    t1 = time.perf_counter()
    i1 = len(dec_end)
    stop.set()
    th.join()
    torch.cuda.synchronize()
    elapsed = t1 - t0
    lo, hi = max(i0, 1) - 1, i1
    tpot = np.array([dec_end[j].elapsed_time(dec_end[j + 1]) for j in range(lo, hi - 1)]) if hi - lo > 2 else np.array([float("nan")])
    steplat = np.array([dec_start[j].elapsed_time(dec_end[j]) for j in range(lo, hi)]) if hi > lo else np.array([float("nan")])
    return {"elapsed": elapsed, "tokens_per_s": K * hz.T / elapsed if finetune else 0.0, "ms_per_step": elapsed * 1e3 / K,
            "tpot": tpot, "steplat": steplat}


class FinetuneFeeder:
    """Host thread that keeps the finetune task running on whatever stream the scheduler last assigned
    (`target`; None = paused).  At most two units are in flight, so a pause or a move to another partition takes
    effect after the unit that is running; a unit on a new stream waits for the last unit on the old one (the
    units share the task's workspace)."""

    def __init__(self, hz):
        self.hz = hz
        self.target = None
        self.units = 0
        self._stop = threading.Event()
        self._evs = []
        self._last_stream = None
        self.error = None
        self.th = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        try:
            torch.cuda.set_device(0)
            while not self._stop.is_set():
                st = self.target
                if st is None:
                    time.sleep(5e-5)
                    continue
                if len(self._evs) >= 2:
                    self._evs[-2].synchronize()
                if self._last_stream is not None and st is not self._last_stream and self._evs:
                    st.wait_event(self._evs[-1])
                self.hz.finetune_unit(st)
                ev = torch.cuda.Event()
                ev.record(st)
                self._evs.append(ev)
                if len(self._evs) > 8:
                    del self._evs[:4]
                self._last_stream = st
                self.units += 1
        except BaseException as e:                 # noqa: BLE001 -- raised again by __exit__
            self.error = e

    def completed(self):
        """Units whose work has finished on the device."""
        pending = sum(0 if e.query() else 1 for e in self._evs[-2:])
        return self.units - pending

    def __enter__(self):
        self.th.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        self.th.join()
        torch.cuda.synchronize()
        self._evs, self._last_stream = [], None    # nothing of this task refers to its streams any more
        if self.error is not None and a[0] is None:
            raise RuntimeError("the finetune thread failed") from self.error


def run_trace(hz, pred, slo_ms, segments, seqlen, refresh_phases=32, starve=(), log=lambda *a: None, feedback=True):
    """Replays a decode load trace under the runtime scheduler (Sec. 6.2) on compute-unit partitions.

    segments: [(phases, batch), ...]; every sequence has `seqlen` cached tokens.  At the beginning of each decode
    phase the library's scheduler decides the partition; decode runs on the first infer_level tenths of the compute
    units, the finetune task on the last ft_level tenths (or not at all).  `starve`: phase indices at which the
    finetune task reports no ready work.  The host waits for each decode step before deciding the next phase.
    Returns per-phase records and a per-segment summary (latency percentiles, share of phases within the target,
    finetune units completed).  feedback: every measured step corrects the predictor at its level by the smoothed ratio
    measured / predicted (`harli_pred_observe`, an addition to the paper's scheduler: Eq. 1 is a straight line in the
    batch size and misses a step on a tenth of the chip by 10 %, enough to pick a plan just above the target); the
    factors are set back to 1 before returning."""
    cs = CuStreams()
    low, high = cs.pairs()
    sched = hb.Scheduler(pred, slo_ms, refresh_phases)
    dev = hz.x_dev.device
    starve = set(starve)
    rec = []
    summary = []
    g = 0
    last_stream, last_ev = None, None
    # made before the finetune task starts: work on the default stream waits for every restricted stream's queue
    lens_of = {bs: torch.full((bs,), seqlen, dtype=torch.int32, device=dev) for _, bs in segments}
    torch.cuda.synchronize()
    with FinetuneFeeder(hz) as feeder:
        for n_ph, bs in segments:
            lens = lens_of[bs]
            u0, t0 = feeder.completed(), time.perf_counter()
            first = len(rec)
            for _ in range(n_ph):
                ready = g not in starve
                i, f, pred_ms, act = sched.step(bs, seqlen, ready)
                feeder.target = high[f] if f > 0 else None
                st = low[i]
                if last_stream is not None and st is not last_stream:
                    st.wait_event(last_ev)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(st)
                hz.decode_launch(st, bs, lens, seqlen + 1)
                e1.record(st)
                e1.synchronize()
                last_stream, last_ev = st, e1
                ms = e0.elapsed_time(e1)
                rec.append({"phase": g, "batch": bs, "infer_level": i, "ft_level": f, "action": act, "predicted_ms": pred_ms,
                            "latency_ms": ms})
                if feedback and pred_ms > 0.0:
                    pred.observe(i, pred_ms / pred.get_scale(i), ms, 0.5)   # the factor has not moved since the plan was made
                g += 1
            dt = time.perf_counter() - t0
            lat = np.array([r["latency_ms"] for r in rec[first:]])
            units = feeder.completed() - u0
            summary.append({"batch": bs, "phases": n_ph, "latency_ms_p50": float(np.percentile(lat, 50)),
                            "latency_ms_p99": float(np.percentile(lat, 99)), "within_slo": float(np.mean(lat <= slo_ms)),
                            "finetune_units": int(units), "finetune_tokens_per_s": units * hz.T / dt,
                            "plans": sorted({(r["infer_level"], r["ft_level"]) for r in rec[first:]}),
                            "replans": int(sum(r["action"] == hb.SCHED_REPLAN for r in rec[first:]))})
            log("[trace] batch %d: %s" % (bs, summary[-1]))
        feeder.target = None
    sched.close()
    scale = [pred.get_scale(lv) for lv in range(1, N_LEVELS + 1)]
    for lv in range(1, N_LEVELS + 1):
        pred.set_scale(lv, 1.0)
    _quiesce(hz)
    cs.close()
    hz.ctx.check(torch.cuda.current_stream())
    return {"phases": rec, "segments": summary, "calibration_by_level": scale}
