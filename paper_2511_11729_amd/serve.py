"""A decode service with continuous batching next to a finetune task, both on one unified pool (Harli Sec. 3-4, the
setting of the evaluation's request trace, Sec. 8.1 / 8.5).  Host orchestration only: every device step runs in
libharli's kernels; this module keeps the request queue, the page tables and the calls in order.

Requests arrive with a prompt whose KV cache is taken as given (the paper serves decode in a prefill/decode
disaggregated deployment: prefill happens elsewhere) and a number of tokens to produce.  Admission allocates the
prompt's KV pages from the pool; every decode step appends one token per running sequence, allocates a page when a
sequence crosses a page boundary and frees the pages of sequences that finish (the pool reuses them once the step
that last read them has completed).  The finetune task allocates its saved activations from the same pool and backs
off when the pool reports pressure or cannot serve it (Sec. 4.4: inference has priority).
"""
from __future__ import annotations

import collections
import threading
import time

import numpy as np
import torch

from . import binding as hb

P = 16  # tokens per KV page


class DecodeServer:
    """Continuous batching over `harli_decode_step`.  Not thread-safe: one thread drives it."""

    def __init__(self, ctx, pool, m, *, max_batch: int, max_len: int, stream, slab=None):
        """slab: the pool's slab as a torch uint8 tensor; when given, the KV pages of an admitted prompt are cleared on
        the decode stream (standing in for the arrival of the prompt's cache from the prefill instance: the same
        bytes are written once).  Without it the pages keep whatever the pool last held there."""
        self.ctx, self.pool, self.m, self.stream = ctx, pool, m, stream
        self.kv_view = None
        if slab is not None:
            cfg, st = pool.cfg, pool.stats()
            page_w = P * cfg.kv_row_bytes // 8         # in 8-byte words: a byte-wise fill is eight times the work
            chunk_w = 2 * cfg.n_layers * cfg.block_bytes // 8
            self.ppb = st.pages_per_block
            self.kv_view = torch.as_strided(slab.view(torch.int64), (st.n_chunks, 2 * cfg.n_layers, self.ppb, page_w),
                                            (chunk_w, cfg.block_bytes // 8, page_w, 1), cfg.small_pool_bytes // 8)
        self.max_batch, self.max_len = max_batch, max_len
        self.max_pages = (max_len + P - 1) // P + 1
        dev = "cuda:0"
        self.table = np.full((max_batch, self.max_pages), -1, np.int32)   # host truth, updated incrementally
        self.kv = np.zeros(max_batch, np.int32)
        self.ring = [(torch.empty(max_batch, self.max_pages, dtype=torch.int32, pin_memory=True),
                      torch.empty(max_batch, dtype=torch.int32, pin_memory=True), None) for _ in range(4)]
        self.table_dev = torch.empty(max_batch, self.max_pages, dtype=torch.int32, device=dev)
        self.kv_dev = torch.empty(max_batch, dtype=torch.int32, device=dev)
        # The per-step uploads go through a stream of torch's own: for a non-blocking copy out of pinned memory torch's
        # host allocator keeps an event on the stream the copy ran on and asks for it when the buffer is freed --
        # possibly after a restricted stream handed in by the caller has been destroyed.
        self.upload = torch.cuda.Stream()
        self.tok = torch.zeros(max_batch, dtype=torch.int32, device=dev)
        with torch.cuda.stream(self.upload):
            self.tok.zero_()                   # first use now, not in the middle of a run
        self.upload.synchronize()
        self.nxt = torch.zeros(max_batch, dtype=torch.int32, device=dev)
        self.logits = torch.empty(max_batch, m.vocab, dtype=torch.float32, device=dev)
        self.x_out = torch.empty(max_batch, m.hidden, dtype=torch.float32, device=dev)
        self.running = []          # per slot: [pages (list), cached tokens, tokens left]
        self.queue = collections.deque()
        self.step_no = 0
        self.last_done = None
        self.admitted = self.finished = self.kv_stalls = self.preempted = self.tokens_out = 0
        self._held = []            # events handed to the pool with freed pages: alive until the pool has polled them
        self.tag = None            # whatever the caller wants kept with the next step (see completed_steps)
        self._timed = collections.deque()
        self._idle = True          # no step was issued at the last call of step(): the next interval starts at its own start

    def use_stream(self, stream):
        """Later steps run on `stream` (a compute-unit partition); they still follow the steps issued so far."""
        if stream is not self.stream:
            if self.last_done is not None:
                stream.wait_event(self.last_done)
            self.stream = stream

    def submit(self, reqs):
        self.queue.extend(reqs)

    def _admit(self):
        while self.queue and len(self.running) < self.max_batch:
            prompt, out = self.queue[0]
            prompt = min(prompt, self.max_len - 2)
            out = max(1, min(out, self.max_len - 1 - prompt))
            need = (prompt + 1 + P - 1) // P
            # headroom: besides the prompt, one more page for every sequence that is running (each reaches a page
            # boundary within 16 steps); without it a pool smaller than the KV demand admits, runs out, sends a
            # sequence back to the queue and admits it again, over and over
            st = self.pool.stats()
            free_pages = (st.kv_chunks + st.free_chunks) * st.pages_per_block - st.kv_pages_live
            if self.running and need + len(self.running) > free_pages:
                self.kv_stalls += 1
                break
            try:
                ids = self.pool.alloc_pages(need)
            except hb.HarliError as e:
                if e.status != hb.HARLI_ERR_OOM:
                    raise
                self.kv_stalls += 1            # no room for this prompt now: it stays queued
                break
            self.queue.popleft()
            if self.kv_view is not None:       # the prompt's cache "arrives": its pages are written once
                # One fill per run of neighbouring pages, on the decode stream, and no index tensor: copying one to the
                # device would make the host wait for every step it has queued, and anything on the default stream
                # would wait for, and hold up, every restricted stream.
                with torch.cuda.stream(self.stream):
                    srt = sorted(ids)
                    k = 0
                    while k < len(srt):
                        c, s0 = divmod(srt[k], self.ppb)
                        j = k + 1
                        while j < len(srt) and srt[j] == srt[j - 1] + 1 and srt[j] // self.ppb == c:
                            j += 1
                        self.kv_view[c, :, s0:s0 + (j - k), :].zero_()
                        k = j
            b = len(self.running)
            self.table[b, :] = -1
            self.table[b, :need] = ids
            self.kv[b] = prompt
            self.running.append([list(ids), prompt, out])
            self.admitted += 1

    def _drop(self, b, event):
        """Frees slot b's pages (reusable once `event` has completed) and moves the last slot into its place."""
        self.pool.free_pages(self.running[b][0], event)
        if event is not None and (not self._held or self._held[-1] is not event):
            self._held.append(event)
        last = len(self.running) - 1
        if b != last:
            self.running[b] = self.running[last]
            self.table[b] = self.table[last]
            self.kv[b] = self.kv[last]
        self.running.pop()

    def step(self):
        """Admits what fits, launches one decode step for every running sequence and advances the host state.
        Returns (event recorded after the step, batch size, event recorded before it) or None when nothing is running."""
        self._admit()
        B = len(self.running)
        if B == 0:
            self._idle = True
            return None
        tb, kb, ev = self.ring[self.step_no % len(self.ring)]
        if ev is not None:
            ev.synchronize()                   # the copy that last used this staging buffer is done
        tb[:B].copy_(torch.from_numpy(self.table[:B]))
        kb[:B].copy_(torch.from_numpy(self.kv[:B]))
        if self.last_done is not None:
            self.upload.wait_event(self.last_done)   # the previous step still reads the device copies
        with torch.cuda.stream(self.upload):
            self.table_dev[:B].copy_(tb[:B], non_blocking=True)
            self.kv_dev[:B].copy_(kb[:B], non_blocking=True)
            up = torch.cuda.Event()
            up.record()
        self.stream.wait_event(up)
        start = torch.cuda.Event(enable_timing=True)
        start.record(self.stream)
        max_kv = int(self.kv[:B].max()) + 1
        self.ctx.decode_step(batch=B, kv_len=self.kv_dev, page_table=self.table_dev, max_pages=self.max_pages, max_kv_len=max_kv,
                             token_ids=self.tok, x_out=self.x_out, logits=self.logits, next_token=self.nxt, stream=self.stream)
        done = torch.cuda.Event(enable_timing=True)
        done.record(self.stream)
        self._timed.append((start if self.last_done is None or self._idle else self.last_done, done, self.tag))
        self._idle = False
        self.last_done = done
        self.ring[self.step_no % len(self.ring)] = (tb, kb, up)
        self.tok, self.nxt = self.nxt, self.tok   # the tokens just produced feed the next step
        self.step_no += 1
        self.tokens_out += B
        if len(self._held) > 256 and self.pool.stats().pending_frees == 0:
            self._held.clear()
        # host state after the step: every sequence holds one more token
        b = 0
        while b < len(self.running):
            seq = self.running[b]
            seq[1] += 1
            seq[2] -= 1
            self.kv[b] = seq[1]
            if seq[2] == 0:
                self._drop(b, done)
                self.finished += 1
                continue                        # slot b now holds another sequence
            if seq[1] + 1 > len(seq[0]) * P:    # the next token starts a new page
                try:
                    pid = self.pool.alloc_pages(1)[0]
                    self.table[b, len(seq[0])] = pid
                    seq[0].append(pid)
                except hb.HarliError as e:
                    if e.status != hb.HARLI_ERR_OOM:
                        raise
                    # the reserve is there to prevent this; if it happens the sequence goes back to the queue
                    self.preempted += 1
                    self.queue.appendleft((seq[1], seq[2]))
                    self._drop(b, done)
                    continue
            b += 1
        return done, B, start

    def completed_steps(self):
        """[(tag, ms)] of the steps that have finished on the device since the last call, oldest first: `tag` is what
        `self.tag` held when the step was issued, ms the time from the end of the step before it to its own end (what a
        request sees as the time per output token: the step itself plus whatever ran on the stream before it, such as
        the arrival of admitted prompts); for the first step, its own time on the device."""
        out = []
        while self._timed and self._timed[0][1].query():
            start, done, tag = self._timed.popleft()
            out.append((tag, start.elapsed_time(done)))
        return out

    def drain(self):
        """Frees every running sequence (end of a run) and lets go of every event recorded on the decode stream, so
        that the caller may destroy that stream afterwards."""
        self.stream.synchronize()
        while self.running:
            self._drop(len(self.running) - 1, None)
        if self.pool.stats().pending_frees == 0:   # the pool has looked at every event it was given
            self._held.clear()
        self.ring = [(tb, kb, None) for tb, kb, _ in self.ring]
        self.last_done = None
        self._timed.clear()


class FinetuneWorker:
    """Host thread stepping a whole-model finetune task.  `step_fn(next_stream)` runs one training step, calling
    `next_stream()` before every layer unit (the paper's scheduling unit, Sec. 6.1) to learn which stream -- which
    compute-unit partition -- the unit goes to; it returns False when the pool could not hold the step.  `target` is the
    stream currently assigned (None: paused; `next_stream` then waits).  Units on a new stream follow the last unit
    on the old one."""

    def __init__(self, pool, step_fn, stream, tokens_per_step):
        self.pool, self.step_fn, self.T = pool, step_fn, tokens_per_step
        self.target = stream
        self.steps = self.oom = self.backoff = self.units = 0
        self.waiting = False            # True while the task has no unit ready to issue (between steps, backing off)
        self.error = None
        self._stop = threading.Event()
        self._last_stream, self._last_ev = None, None
        self.th = threading.Thread(target=self._run, daemon=True)

    def next_stream(self):
        while True:
            st = self.target
            if st is not None or self._stop.is_set():
                break
            time.sleep(1e-4)
        if st is None:
            st = self._last_stream or torch.cuda.current_stream()
        if self._last_ev is not None and st is not self._last_stream:
            st.wait_event(self._last_ev)
        return st

    def unit_done(self, st):
        """Called by step_fn after it has enqueued a unit on `st`: at most two units are in flight, so that a change of
        partition or a pause takes effect within about one unit."""
        ev = torch.cuda.Event()
        ev.record(st)
        prev = self._last_ev
        self._last_stream, self._last_ev = st, ev
        self.units += 1
        if prev is not None:
            prev.synchronize()

    def _run(self):
        try:
            torch.cuda.set_device(0)
            while not self._stop.is_set():
                if self.pool.pressure() > 0:   # inference needs the memory (Sec. 4.4): do not start a step now
                    self.backoff += 1
                    self.waiting = True
                    time.sleep(2e-3)
                    continue
                self.waiting = False
                ok = self.step_fn(self)
                if ok:
                    self.steps += 1
                else:
                    self.oom += 1
                    self.waiting = True
                    time.sleep(2e-3)
        except BaseException as e:             # noqa: BLE001 -- raised again by __exit__
            self.error = e
            self.waiting = True

    def __enter__(self):
        self.th.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        self.th.join()
        torch.cuda.synchronize()
        self._last_stream, self._last_ev = None, None
        if self.error is not None and a[0] is None:
            raise RuntimeError("the finetune thread failed") from self.error


def replay(server: DecodeServer, arrivals, worker_factory=None, slo_ms=40.0, sample_every=25, log=lambda *a: None, plan=None):
    """Drives `server` through `arrivals` (one list of requests per decode step) with, optionally, a finetune worker
    beside it.  `plan(server, worker)`, when given, is called at the beginning of every decode phase (Sec. 6.2) and may
    move the two tasks to other streams or pause the finetune task; it returns a record that is kept with the step.
    Returns counters, pool snapshots and, per decode step, the batch size, the plan's record and the time per output
    token (`tpot_ms[k]` is the time from the end of step k to the end of step k + 1; `step_ms[k]` is step k's own time
    on the device, from its first kernel to its last)."""
    pool = server.pool
    recs, snaps, plans = [], [], []
    t_start = time.perf_counter()
    box = {"worker": None}

    def run():
        pending = collections.deque()
        for t, reqs in enumerate(arrivals):
            server.submit(reqs)
            decided = plan(server, box["worker"]) if plan is not None else None
            r = server.step()
            if r is not None:
                pending.append(r)
                recs.append(r)
                plans.append(decided)
            if len(pending) > 2:
                pending.popleft()[0].synchronize()     # the host runs at most two steps ahead of the device
            if t % sample_every == 0:
                st = pool.stats()
                snaps.append({"step": t, "batch": len(server.running), "queued": len(server.queue), "free_chunks": st.free_chunks,
                              "kv_chunks": st.kv_chunks, "tensor_chunks": st.tensor_chunks,
                              "pressure": pool.pressure()})
            if t % 200 == 0:
                log("[serve] step %d of %d: batch %d, queued %d, %.1f s" % (t, len(arrivals), len(server.running), len(server.queue),
                                                                       time.perf_counter() - t_start))
        server.stream.synchronize()

    if worker_factory is not None:
        with worker_factory() as worker:
            box["worker"] = worker
            run()
        ft = {"steps": worker.steps, "oom_retries": worker.oom, "pressure_backoffs": worker.backoff, "tokens": worker.steps * worker.T}
    else:
        run()
        ft = None
    elapsed = time.perf_counter() - t_start
    tpot = np.array([recs[i][0].elapsed_time(recs[i + 1][0]) for i in range(len(recs) - 1)]) if len(recs) > 1 else np.array([0.0])
    batches = np.array([r[1] for r in recs])
    busy = np.array([r[2].elapsed_time(r[0]) for r in recs]) if recs else np.array([0.0])
    out = {"steps": len(arrivals), "decode_steps": len(recs), "elapsed_s": elapsed, "tokens_out": server.tokens_out,
           "decode_tokens_per_s": server.tokens_out / elapsed, "tpot_ms_p50": float(np.percentile(tpot, 50)),
           "tpot_ms_p99": float(np.percentile(tpot, 99)), "tpot_ms_max": float(tpot.max()), "within_slo": float(np.mean(tpot <= slo_ms)),
           "batch_mean": float(batches.mean()) if len(batches) else 0.0, "batch_max": int(batches.max()) if len(batches) else 0,
           "admitted": server.admitted, "finished": server.finished, "kv_admission_stalls": server.kv_stalls,
           "preempted": server.preempted, "queued_at_end": len(server.queue), "snapshots": snaps,
           "plans": plans if plan is not None else [], "tpot_ms": tpot, "batches": batches, "step_ms": busy}
    if ft is not None:
        ft["tokens_per_s"] = ft["tokens"] / elapsed
        out["finetune"] = ft
    return out
