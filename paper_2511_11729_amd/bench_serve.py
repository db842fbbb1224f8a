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

    def ft_step(st):
        """One training step; False when the pool could not hold the step's activations (everything taken is returned)."""
        with torch.cuda.stream(st):
            torch.index_select(embf, 0, tok_dev, out=acts[0])
        saved = []
        try:
            for l in range(L):
                saved.append(ctx.lora_fwd(l, acts[l], acts[l + 1], ft.micro_batch, ft.seq_len, stream=st))
        except hb.HarliError as e:
            if e.status != hb.HARLI_ERR_OOM:
                raise
            for sv in saved:
                ctx.saved_release(sv, stream=st)
            st.synchronize()
            return False
        state["t"] += 1
        ctx.head_fwd_bwd(acts[L], tg_dev, loss, d0, stream=st)
        d, dn = d0, d1
        for l in range(L - 1, -1, -1):
            ctx.lora_bwd(l, d, dn, saved[l], dA[l], dB[l], stream=st)
            d, dn = dn, d
        for l in range(L):
            for p in A[l]:
                hb.adamw_step(masters[l][p][0], moms[l][p][0], moms[l][p][1], dA[l][p], A[l][p], step=state["t"], lr=1e-4,
                              zero_grad=True, stream=st)
                hb.adamw_step(masters[l][p][1], moms[l][p][2], moms[l][p][3], dB[l][p], Bm[l][p], step=state["t"], lr=1e-4,
                              zero_grad=True, stream=st)
        st.synchronize()
        return True

    keep = (slab, layer, emb, gf, wlm, A, Bm, acts, masters, moms, dA, dB, embf, tok_dev, tg_dev, d0, d1, loss)
    return w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep


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
    args = ap.parse_args()

    import torch
    import workloads as wl
    from paper_2511_11729_amd import serve

    w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep = build(args)
    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()
    server = serve.DecodeServer(ctx, pool, m, max_batch=args.max_batch, max_len=args.max_len, stream=sD, slab=keep[0])
    arrivals = wl.make_arrivals(w, args.steps, tuple(args.targets), args.mean_out,
                                prompt=w.decode.len_dist if w.decode.len_dist[0] == "lognormal" else ("lognormal", 800, 0.6, 8192))
    arrivals = [[(min(p, args.max_len - 2), o) for p, o in reqs] for reqs in arrivals]
    factory = None if args.no_finetune else (lambda: serve.FinetuneWorker(pool, ft_step, sF, ft.tokens))
    res = serve.replay(server, arrivals, factory, slo_ms=args.slo_ms, log=lambda *a: print(*a, file=sys.stderr, flush=True))
    server.drain()
    ctx.check(sD)
    st = pool.stats()
    res["workload"] = ("config %d, %d layers + output layer: arrival trace with steady-state batches %s over %d decode steps, mean "
                       "output %d tokens; finetune %d x %d tokens per step" % (args.config, m.n_layers, args.targets, args.steps,
                                                                             args.mean_out, ft.micro_batch, ft.seq_len))
    res["pool"] = {"chunks": n_chunks, "chunk_MB": chunk / 1e6, "slab_GB": slab_bytes / 1e9, "reserve_chunks": reserve,
                   "kv_pages_live_at_end": st.kv_pages_live, "tensor_blocks_live_at_end": st.tensor_blocks_live}
    res["slo_tpot_ms"] = args.slo_ms
    snaps = res.pop("snapshots")
    res["pool_census"] = snaps[:: max(1, len(snaps) // 24)]
    print(json.dumps(res))


if __name__ == "__main__":
    main()
