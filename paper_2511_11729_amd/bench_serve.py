"""A request trace served next to a finetune task on one unified pool:  python -m paper_2511_11729_amd.bench_serve --config 4

The decode instance runs continuous batching over a synthetic arrival trace (piecewise-constant Poisson rates whose
steady-state batch sizes cycle through 1, 8, 42, 24, 128, 256 -- 8 / 42 / 24 are the light / heavy / medium loads of the
paper's controlled experiment, Sec. 8.5 -- log-normal prompt lengths, geometric output lengths; prompts arrive with
their KV cache, as from a separate prefill instance).  KV pages are allocated and freed as sequences start, grow and
finish.  Beside it the finetune instance steps the whole model (LoRA forward, output layer + cross entropy, backward,
AdamW) and takes its saved activations from the SAME pool, backing off when the pool reports pressure or cannot serve
it.  Prints one JSON line: time per output token (p50 / p99 / max, share of steps inside the target), decode and
finetune tokens/s, admission stalls, pre-emptions, finetune out-of-memory retries and the pool's chunk census over
time.  --pool-gb sizes the slab: roomy by default, tight to exercise the coordination.

--sched profiles the latency predictor on compute-unit partitions first (Sec. 5: Eq. 1 per level on the whole model,
Eq. 2 beside whole training steps) and then lets the runtime scheduler (Sec. 6.2) place both tasks at the beginning of
every decode phase: decode on the first tenths of the compute units, the finetune task's next layer unit on the last
tenths, or paused.  The plan hook also times the finished steps and folds measured / predicted back into the predictor
per level (--no-feedback: the profiled predictor alone).  Comparators: --static I F (one partition throughout, the
shape of the paper's StaticMode), --ft-all-cus (only the inference partition enforced).  --dump writes one CSV row per
decode step (batch, plan, predicted and measured times).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def build(args, model=None):
    import dataclasses
    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb
    from paper_2511_11729_amd.harness import dev_bf16, dev_f32

    hb.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.workload(args.config)
    kw = {}
    if args.layers is not None:
        kw["n_layers"] = args.layers
    if args.vocab is not None:
        kw["vocab"] = args.vocab
    m = model if model is not None else (dataclasses.replace(w.model, **kw) if kw else w.model)
    if m.dtype != "bf16" or m.vocab <= 0:
        raise SystemExit("bench_serve: needs a bf16 workload with an output layer (configs 2-5)")
    w = dataclasses.replace(w, model=m)
    ft = w.finetune if args.ft_tokens is None else wl.FinetuneCfg(args.ft_tokens[0], args.ft_tokens[1], "ce")
    lora = w.lora
    L, T, H = m.n_layers, ft.tokens, m.hidden

    W_np = wl.make_layer_weights(w, 0, m)
    ex = wl.make_model_extras(w, m)
    layer = {n: dev_bf16(W_np[n]) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
    layer["g1"], layer["g2"] = dev_f32(W_np["g1"]), dev_f32(W_np["g2"])
    for bn in ("bq", "bk", "bv"):
        if bn in W_np:
            layer[bn] = dev_f32(W_np[bn])
    emb, gf, wlm = dev_bf16(ex["emb"]), dev_f32(ex["gf"]), dev_bf16(ex["wlm"])
    lora_np = wl.make_lora(w, 0, m, lora)
    A = [{p: dev_bf16(a) for p, (a, b) in lora_np.items()} for _ in range(L)]
    Bm = [{p: dev_bf16(b) for p, (a, b) in lora_np.items()} for _ in range(L)]

    block = 2 << 20
    chunk = L * 2 * block
    per_layer = T * H * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6
    act_chunks = (L + 1) * (per_layer // chunk + 2) + 4
    small = 256 << 20
    if args.pool_gb is not None:
        n_chunks = max(4, int((args.pool_gb * 1e9 - small) // chunk))
    else:                                                 # roomy: the largest phase's KV cache plus a whole step's activations
        kv_tokens = args.max_batch * min(args.max_len, 1400)
        n_chunks = -(-kv_tokens * 2 * m.kv_row_bytes * L // chunk) + act_chunks + 8
        if getattr(args, "window", None):             # the window's slots are pool memory too
            n_chunks += min(args.window, 2 * L) * (-(-2 * m.layer_params // chunk) + 1)
    slab_bytes = small + n_chunks * chunk
    slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=dev)
    pool = hb.Pool(slab, slab_bytes, block_bytes=block, n_layers=L, kv_row_bytes=m.kv_row_bytes, small_pool_bytes=small,
                   kv_reserve_chunks=1)
    # Sec. 4.4: keep what decode can ask for while the finetune task gives memory back (about one layer unit)
    reserve = pool.reserve_chunks_for(args.release_ms, args.slo_ms, args.max_batch)
    pool.set_reserve(reserve)
    ctx = hb.Context(pool, n_layers=L, hidden=H, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim, ffn=m.ffn,
                     vocab=m.vocab, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=args.max_batch,
                     max_seq_len=args.max_len + 8, max_ft_tokens=T, layers=[layer] * L, emb=emb, g_final=gf, w_lm=wlm)
    ctx.lora_attach(lora.rank, lora.alpha, lora.targets, A, Bm)

    tok = wl.make_token_ids(w, (ft.micro_batch, ft.seq_len)) % m.vocab
    tg = np.full(tok.shape, -1, np.int32)
    tg[:, :-1] = tok[:, 1:]
    tok_dev = torch.from_numpy(tok.reshape(-1).astype(np.int64)).to(dev)
    tg_dev = torch.from_numpy(tg.reshape(-1)).to(dev)
    acts = [torch.empty(T, H, dtype=torch.float32, device=dev) for _ in range(L + 1)]
    d0, d1 = torch.empty(T, H, device=dev), torch.empty(T, H, device=dev)
    loss = torch.zeros(1, device=dev)
    masters = [{p: (A[l][p].float(), Bm[l][p].float()) for p in A[l]} for l in range(L)]
    moms = [{p: [torch.zeros_like(masters[l][p][0]), torch.zeros_like(masters[l][p][0]), torch.zeros_like(masters[l][p][1]),
                 torch.zeros_like(masters[l][p][1])] for p in A[l]} for l in range(L)]
    dA = [{p: torch.zeros_like(masters[l][p][0]) for p in A[l]} for l in range(L)]
    dB = [{p: torch.zeros_like(masters[l][p][1]) for p in A[l]} for l in range(L)]
    embf = emb.float()
    state = {"t": 0}

    def ft_step(wk):
        """One training step, unit by unit: before each unit `wk.next_stream()` names the stream (compute-unit partition) it
        goes to.  False when the pool could not hold the step's activations (everything taken is returned)."""
        st = wk.next_stream()
        with torch.cuda.stream(st):
            torch.index_select(embf, 0, tok_dev, out=acts[0])
        wk.unit_done(st)
        saved = []
        try:
            for l in range(L):
                st = wk.next_stream()
                saved.append(ctx.lora_fwd(l, acts[l], acts[l + 1], ft.micro_batch, ft.seq_len, stream=st))
                wk.unit_done(st)
        except hb.HarliError as e:
            if e.status != hb.HARLI_ERR_OOM:
                raise
            for sv in saved:
                ctx.saved_release(sv, stream=st)
            st.synchronize()
            return False
        state["t"] += 1
        st = wk.next_stream()
        ctx.head_fwd_bwd(acts[L], tg_dev, loss, d0, stream=st)
        wk.unit_done(st)
        d, dn = d0, d1
        for l in range(L - 1, -1, -1):
            st = wk.next_stream()
            ctx.lora_bwd(l, d, dn, saved[l], dA[l], dB[l], stream=st)
            wk.unit_done(st)
            d, dn = dn, d
        st = wk.next_stream()
        for l in range(L):
            for p in A[l]:
                hb.adamw_step(masters[l][p][0], moms[l][p][0], moms[l][p][1], dA[l][p], A[l][p], step=state["t"], lr=1e-4,
                              zero_grad=True, stream=st)
                hb.adamw_step(masters[l][p][1], moms[l][p][2], moms[l][p][3], dB[l][p], Bm[l][p], step=state["t"], lr=1e-4,
                              zero_grad=True, stream=st)
        wk.unit_done(st)
        st.synchronize()
        return True

    keep = (slab, layer, emb, gf, wlm, A, Bm, acts, masters, moms, dA, dB, embf, tok_dev, tg_dev, d0, d1, loss)
    return w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep


def make_plan(args, m, ft, pool, ctx, ft_step, server, log):
    """Profiles whole-model decode on compute-unit partitions (alone, then with training steps beside it), fits the
    predictor and returns the per-phase planning hook for serve.replay."""
    import torch
    from paper_2511_11729_amd import binding as hb
    from paper_2511_11729_amd import colocate, serve

    dev = "cuda:0"
    PN = min(1536, args.max_len - 8)
    pages_per = (PN + 1 + serve.P - 1) // serve.P
    # the largest profiled batch whose KV cache fits beside a training step's activations (a tight pool profiles less)
    st = pool.stats()
    L = m.n_layers
    chunk = 2 * L * pool.cfg.block_bytes
    saved = ctx.saved_bytes(ft.micro_batch, ft.seq_len)                   # what one layer's forward keeps for its backward
    room = st.free_chunks - (L * (-(-saved // chunk) + 1) + 8)
    PB = next((b for b in (160, 128, 96, 64, 32, 16) if b <= args.max_batch and -(-b * pages_per // st.pages_per_block) <= room), None)
    if PB is None:
        raise SystemExit("bench_serve: the pool is too small to profile the predictor beside a training step")
    ids = pool.alloc_pages(PB * pages_per)
    table = torch.full((PB, server.max_pages), -1, dtype=torch.int32, device=dev)
    table[:, :pages_per] = torch.tensor(ids, dtype=torch.int32).reshape(PB, pages_per).to(dev)
    tok = torch.zeros(PB, dtype=torch.int32, device=dev)
    rep_b, rep_n = min(32, PB), min(1024, PN)       # the representative batch of the co-located samples
    rep_kv = torch.full((rep_b,), rep_n, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    class Fixed:                                    # a training step pinned to one stream
        def __init__(self, st):
            self.st = st

        def next_stream(self):
            return self.st

        def unit_done(self, st):
            pass

    class Hz:
        x_dev = tok
        T = ft.tokens

        def decode_launch(self, stream, batch, kv_len_dev, max_kv):
            if batch is None:                       # nothing here may touch the default stream (it would wait for the
                batch, max_kv, kv_len_dev = rep_b, rep_n + 1, rep_kv       # finetune stream's queue)
            ctx.decode_step(batch=batch, kv_len=kv_len_dev, page_table=table, max_pages=server.max_pages, max_kv_len=max_kv,
                            token_ids=tok, x_out=server.x_out, logits=server.logits, next_token=server.nxt, stream=stream)

        def finetune_unit(self, stream):
            ft_step(Fixed(stream))

    grid_b = tuple(b for b in (4, 16, 32, 64, 160) if b <= PB)   # two or three per kernel family of the decode step
    grid_n = tuple(n for n in (128, 512, 1024, 1536) if n <= PN)
    held = tuple((b, n) for b, n in ((8, 256), (24, 768), (96, 1280)) if b <= PB and n <= PN)
    pred, rep = colocate.profile(Hz(), steps=3, log=log, batches=grid_b, seqlens=grid_n, heldout=held)
    pool.free_pages(ids)
    log("[sched] decode alone by level (ms): " + " ".join("%.1f" % v for v in rep["solo_ms_by_level_workload_batch"]))
    log("[sched] decode beside finetune (ms): " + " ".join("%s=%.1f" % kv for kv in rep["colo_ms"].items()))
    rep = {k: rep[k] for k in ("eq1_mean_abs_err_fitted_points", "eq1_mean_abs_err_heldout", "eq1_batch_split",
                               "eq1_as_printed_mean_abs_err_fitted_points", "eq1_as_printed_mean_abs_err_heldout", "eq2_b1_k1", "eq2_mean_abs_err")}
    cs = colocate.CuStreams()
    low, high = cs.pairs(log)
    ft_all = None
    if args.ft_all_cus:                              # only inference is confined; the finetune task may use every compute unit
        ft_all = cs.unrestricted
        if ft_all is None:
            raise SystemExit("bench_serve: no ordinary stream off the inference streams' dispatch pipes was found")
    sched = hb.Scheduler(pred, args.slo_ms * args.sched_margin, 64)

    scale = [1.0] * (colocate.N_LEVELS + 1)         # per level (index 0 unused): the predictor's factors, for the report

    def calibrate(srv):
        """Sec. 6.2 plans with the predictor alone; here the steps that have finished are timed and the ratio
        measured / predicted is folded back into the predictor per level (harli_pred_observe; --no-feedback: off).  It
        absorbs what Eq. 1 cannot hold: latency that is a staircase in the batch size, batches of mixed lengths."""
        n = 0
        for tag, ms in srv.completed_steps():
            if tag is None or tag[1] <= 0.0:
                continue
            pred.observe(tag[0], tag[1], ms, 0.15)
            n += 1
        if n:
            scale[1:] = [pred.get_scale(j) for j in range(1, colocate.N_LEVELS + 1)]

    def plan(srv, worker):
        if not args.no_feedback:
            calibrate(srv)
        B = min(args.max_batch, len(srv.running) + len(srv.queue))
        if B == 0:
            srv.tag = None
            return (colocate.N_LEVELS, 0, -1, 0.0, 0)
        n = int(srv.kv[: max(1, len(srv.running))].mean()) if srv.running else 800
        ready = worker is not None and not worker.waiting
        if args.static is not None:                 # StaticMode-style comparator (Sec. 8.1): one partition throughout
            i, f = args.static
            pred_ms, act = pred.colo(i, f, B, n) if f > 0 else pred.solo(i, B, n), 0
        else:
            i, f, pred_ms, act = sched.step(B, n, ready)
        srv.use_stream(low[i])
        srv.tag = (i, pred_ms / pred.get_scale(i))  # the prediction before calibration
        if worker is not None:
            worker.target = (ft_all if ft_all is not None else high[f]) if f > 0 else None
        return (i, f, act, pred_ms, n)

    rep["planned_for_ms"] = args.slo_ms * args.sched_margin
    rep["feedback"] = not args.no_feedback
    rep["calibration_by_level"] = scale              # filled in as the run goes (read after it)
    return plan, rep, cs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--layers", type=int, default=None, help="depth override")
    ap.add_argument("--vocab", type=int, default=None, help="vocabulary override")
    ap.add_argument("--steps", type=int, default=1800, help="decode steps of the trace")
    ap.add_argument("--targets", type=int, nargs="+", default=[1, 8, 42, 24, 128, 256], help="steady-state batch sizes, in turn")
    ap.add_argument("--mean-out", type=int, default=256, help="mean output length (tokens)")
    ap.add_argument("--max-batch", type=int, default=256)
    ap.add_argument("--max-len", type=int, default=8192 + 1024)
    ap.add_argument("--ft-tokens", type=int, nargs=2, default=None, metavar=("SEQS", "LEN"), help="finetune micro-batch override")
    ap.add_argument("--pool-gb", type=float, default=None, help="slab size; default: roomy")
    ap.add_argument("--slo-ms", type=float, default=40.0)
    ap.add_argument("--release-ms", type=float, default=12.0, help="time the finetune task needs to give memory back")
    ap.add_argument("--no-finetune", action="store_true")
    ap.add_argument("--window", type=int, default=None, metavar="SLOTS",
                    help="keep the finetune task's frozen weights on the host and at most SLOTS of the 2 x layers copies in the "
                         "pool (Sec. 4.3); between steps the window shrinks when inference needs memory and grows again when "
                         "chunks are free (Sec. 4.4)")
    ap.add_argument("--sched", action="store_true",
                    help="profile the latency predictor on compute-unit partitions first, then let the runtime scheduler "
                         "place both tasks at the beginning of every decode phase (Sec. 5, Sec. 6.2)")
    ap.add_argument("--static", type=int, nargs=2, default=None, metavar=("I", "F"),
                    help="with --sched: no runtime scheduling, inference on the first I tenths of the compute units and the "
                         "finetune task on the last F tenths (0: paused) throughout")
    ap.add_argument("--ft-all-cus", action="store_true",
                    help="with --sched: only the inference partition is enforced; finetune units run on every compute unit "
                         "(outside the paper's disjoint plans; the decode step is then slower than the profile says and "
                         "the calibration takes that up)")
    ap.add_argument("--no-feedback", action="store_true",
                    help="with --sched: plan with the profiled predictor alone, without folding measured step times back in")
    ap.add_argument("--dump", default=None, help="with --sched: per-step records (batch, plan, predicted and measured times) as CSV")
    ap.add_argument("--sched-margin", type=float, default=0.9, help="the scheduler plans for this fraction of the target")
    args = ap.parse_args()

    import faulthandler
    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb
    from paper_2511_11729_amd import serve

    faulthandler.enable()                           # a crash in native code names the Python line it came from
    w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep = build(args)
    scheduled = args.sched and not args.no_finetune
    sD = torch.cuda.Stream()
    sF = None if scheduled else torch.cuda.Stream()          # scheduled: the plan names the finetune stream, phase by phase
    with torch.cuda.stream(sD):
        keep[-1].zero_()                             # first use of the stream now (its hardware queue is set up here)
    sD.synchronize()
    server = serve.DecodeServer(ctx, pool, m, max_batch=args.max_batch, max_len=args.max_len, stream=sD, slab=keep[0])
    arrivals = wl.make_arrivals(w, args.steps, tuple(args.targets), args.mean_out,
                                prompt=w.decode.len_dist if w.decode.len_dist[0] == "lognormal" else ("lognormal", 800, 0.6, 8192))
    arrivals = [[(min(p, args.max_len - 2), o) for p, o in reqs] for reqs in arrivals]
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    step_fn, window_log = ft_step, []
    if args.window is not None and not args.no_finetune:
        # Sec. 4.3 / 4.4: the finetune task's frozen weights live on the host and only a window of them in the pool;
        # between training steps the window gives slots back when inference needs the memory and takes slots again when
        # chunks are free.  (No finetune unit is in flight between steps: ft_step ends with a wait for its stream.)
        L2 = 2 * m.n_layers
        ctx.ft_window_enable(min(args.window, L2))
        ws0 = ctx.ft_window_stats()
        slot_chunks = -(-ws0.slot_bytes // chunk)
        log("[window] %d of %d slots of %.0f MB on the device" % (ws0.slots, L2, ws0.slot_bytes / 1e6))
        state = {"oom": False, "calm": 0}
        saved = ctx.saved_bytes(ft.micro_batch, ft.seq_len)               # what one layer's forward keeps for its backward
        need = m.n_layers * (-(-saved // chunk) + 1) + reserve + 8          # a step's saved activations, the KV reserve, slack
        top = min(args.window, L2)

        def step_fn(wk):
            ws, st = ctx.ft_window_stats(), pool.stats()
            target, state["calm"] = hb.ft_window_advise(ws.slots, max(top, ws.slots), slot_chunks, st.free_chunks, need,
                                                        pool.pressure() > 0 or state["oom"], state["calm"])
            if target != ws.slots:
                try:
                    ctx.ft_window_resize(target)
                except hb.HarliError as e:
                    if e.status != hb.HARLI_ERR_OOM:
                        raise
                window_log.append({"decode_step": server.step_no, "slots": ctx.ft_window_stats().slots,
                                   "free_chunks": pool.stats().free_chunks})
            ok = ft_step(wk)
            state["oom"] = not ok
            return ok

    factory = None if args.no_finetune else (lambda: serve.FinetuneWorker(pool, step_fn, sF, ft.tokens))
    plan, sched_report, cs = None, None, None
    if scheduled:
        if args.window is not None:                 # the profile needs a training step's activations and a KV cache of its own
            while pool.stats().free_chunks < need + 110 and ctx.ft_window_stats().slots > 4:
                ctx.ft_window_resize(ctx.ft_window_stats().slots - 4)
            log("[window] %d slots while the predictor is profiled" % ctx.ft_window_stats().slots)
        plan, sched_report, cs = make_plan(args, m, ft, pool, ctx, ft_step, server, log)
    import gc
    gc.collect()
    gc.freeze()                                     # a full collection over the set-up's objects stops the host for ~20 ms
    res = serve.replay(server, arrivals, factory, slo_ms=args.slo_ms, log=log, plan=plan)
    server.drain()
    server.use_stream(sD)
    ctx.check(sD)
    if cs is not None:
        cs.close()                                  # only now: no event and no task refers to the restricted streams any more
    plans, tpot, batches, busy = res.pop("plans"), res.pop("tpot_ms"), res.pop("batches"), res.pop("step_ms")
    res["step_ms_p50"], res["step_ms_p99"] = float(np.percentile(busy, 50)), float(np.percentile(busy, 99))
    if plans and args.dump:
        with open(args.dump, "w") as fh:
            fh.write("step,batch,mean_len,infer_level,ft_level,predicted_ms,tpot_ms,step_ms\n")
            for k in range(1, len(plans)):
                fh.write("%d,%d,%d,%d,%d,%.3f,%.3f,%.3f\n" % (k, batches[k], plans[k][4], plans[k][0], plans[k][1], plans[k][3],
                                                          tpot[k - 1], busy[k]))
    if plans:
        by = {}
        for k in range(1, len(plans)):              # tpot[k - 1] is the duration of decode step k
            i, f, act, pred_ms = plans[k][:4]
            by.setdefault((i, f), []).append((tpot[k - 1], pred_ms, batches[k], busy[k]))
        rows = []
        for (i, f), v in sorted(by.items(), key=lambda kv: -len(kv[1]))[:10]:
            v = np.array(v)
            rows.append({"infer_level": i, "ft_level": f, "phases": len(v), "batch_mean": float(v[:, 2].mean()),
                         "tpot_ms_mean": float(v[:, 0].mean()), "tpot_ms_p10_p50_p90": [float(x) for x in np.percentile(v[:, 0], (10, 50, 90))],
                         "step_ms_mean": float(v[:, 3].mean()), "predicted_ms_mean": float(v[:, 1].mean()),
                         "within_slo": float(np.mean(v[:, 0] <= args.slo_ms))})
        res["scheduler"] = dict(sched_report, plans_used=rows, replans=sum(p[2] == 1 for p in plans),
                                starved_phases=sum(p[2] == 3 for p in plans), paused_phases=sum(p[2] == 2 for p in plans))
    st = pool.stats()
    res["workload"] = ("config %d, %d layers + output layer: arrival trace with steady-state batches %s over %d decode steps, mean "
                       "output %d tokens; finetune %d x %d tokens per step" % (args.config, m.n_layers, args.targets, args.steps,
                                                                             args.mean_out, ft.micro_batch, ft.seq_len))
    res["pool"] = {"chunks": n_chunks, "chunk_MB": chunk / 1e6, "slab_GB": slab_bytes / 1e9, "reserve_chunks": reserve,
                   "kv_pages_live_at_end": st.kv_pages_live, "tensor_blocks_live_at_end": st.tensor_blocks_live}
    res["slo_tpot_ms"] = args.slo_ms
    if args.window is not None and not args.no_finetune:
        ws = ctx.ft_window_stats()
        res["window"] = {"slots_at_start": ws0.slots, "slots_at_end": ws.slots, "slot_MB": ws.slot_bytes / 1e6,
                         "host_GB": ws.host_bytes / 1e9, "h2d_GB": ws.h2d_bytes / 1e9, "hits": ws.hits, "misses": ws.misses,
                         "refills": ws.refills, "resizes": window_log[:: max(1, len(window_log) // 40)]}
    snaps = res.pop("snapshots")
    res["pool_census"] = snaps[:: max(1, len(snaps) // 24)]
    print(json.dumps(res))


if __name__ == "__main__":
    main()
