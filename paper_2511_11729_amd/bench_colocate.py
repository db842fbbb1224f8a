"""Full-depth co-location on one GPU:  python -m paper_2511_11729_amd.bench_colocate --config 2

The paper's own setting at the scale it evaluates (Sec. 8: one model served, the same model finetuned): an inference
instance decoding a whole model (embedding, every layer, output layer, argmax; one HIP graph per step, replayed by a
host thread on stream D) next to a finetune instance stepping the whole model (every layer's LoRA forward, output
layer with next-token cross entropy, every layer's backward, AdamW on every adapter; stream F).  Both instances keep
their own device copies of the frozen weights (Sec. 7) and draw KV pages and saved activations from ONE unified pool.
Seeded random weights (all layers share one host-generated set; the device copies are per layer).  Prints one JSON
line: solo numbers of both tasks, then the co-located run -- finetune tokens/s, decode time per output token (p50,
p99, share of steps inside the target) -- with decode back to back and with decode paced at a request rate.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--layers", type=int, default=None, help="depth override")
    ap.add_argument("--batch", type=int, default=None, help="decode batch (default: the workload's)")
    ap.add_argument("--kv-len", type=int, default=None, help="cached tokens per sequence (default: the workload's draw)")
    ap.add_argument("--steps", type=int, default=4, help="timed finetune steps per run")
    ap.add_argument("--slo-ms", type=float, default=40.0, help="decode time-per-output-token target")
    ap.add_argument("--pace-ms", type=float, default=None, help="paced run: one decode step every this many ms (default 0.6 x target)")
    args = ap.parse_args()
    print(json.dumps(run(args)))


def run(args):
    """The measurement itself; `args` carries config, layers, batch, kv_len, steps, slo_ms, pace_ms.  Returns the
    result dictionary (bench.py calls this for its full-depth leg)."""
    import dataclasses
    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb
    from paper_2511_11729_amd import colocate
    from paper_2511_11729_amd.harness import dev_bf16, dev_f32

    hb.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.workload(args.config)
    m = w.model if args.layers is None else dataclasses.replace(w.model, n_layers=args.layers)
    if m.dtype != "bf16" or m.vocab <= 0:
        raise SystemExit("bench_colocate: needs a bf16 workload with an output layer (configs 2-5)")
    ft, lora = w.finetune, w.lora
    L, T, H, P = m.n_layers, ft.tokens, m.hidden, 16
    B = args.batch or w.decode.batch
    kv_len = (np.full(B, args.kv_len, np.int32) if args.kv_len is not None else wl.draw_lengths(w, B)).astype(np.int32)

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

    # ---- one pool for the KV cache of the decode batch and the saved activations of the finetune step
    block = 2 << 20
    chunk = L * 2 * block
    ppb = block // (P * m.kv_row_bytes)
    n_pages = [(int(n) + 1 + P - 1) // P for n in kv_len]
    total_pages = sum(n_pages)
    per_layer = T * H * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6
    kv_chunks = -(-total_pages // ppb) + 1
    # the library's own memory (decode weight copies, the finetune instance's two copies per layer, the output layer's
    # copies, both workspaces) is taken from the same pool
    lib_bytes = 6 * m.layer_params * L + 6 * m.vocab * H + 6 * T * m.vocab + 4 * per_layer + (2 << 30)
    # (a third more than the bytes: matrices larger than a chunk take runs of adjacent chunks and leave gaps)
    n_chunks = kv_chunks + (L + 1) * (per_layer // chunk + 2) + lib_bytes * 4 // (3 * chunk) + 8
    small = 256 << 20
    slab_bytes = small + n_chunks * chunk
    slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=dev)
    pool = hb.Pool(slab, slab_bytes, block_bytes=block, n_layers=L, kv_row_bytes=m.kv_row_bytes, small_pool_bytes=small,
                   kv_reserve_chunks=1)
    ids = np.array(pool.alloc_pages(total_pages), np.int64)[wl.page_order(w, total_pages)]
    max_pages = max(n_pages) + 1
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :n_pages[b]] = ids[k:k + n_pages[b]]
        k += n_pages[b]
    ctx = hb.Context(pool, n_layers=L, hidden=H, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim, ffn=m.ffn,
                     vocab=m.vocab, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=B,
                     max_seq_len=int(kv_len.max()) + 8, max_ft_tokens=T, layers=[layer] * L, emb=emb, g_final=gf, w_lm=wlm,
                     memory_in_pool=True)
    ctx.lora_attach(lora.rank, lora.alpha, lora.targets, A, Bm)

    # ---- decode instance
    kv_dev = torch.from_numpy(kv_len).to(dev)
    table_dev = torch.from_numpy(table).to(dev)
    tok1 = torch.from_numpy(wl.make_token_ids(w, (B,)).astype(np.int32)).to(dev)
    logits = torch.empty(B, m.vocab, dtype=torch.float32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    x_out = torch.empty(B, H, dtype=torch.float32, device=dev)
    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()

    def decode_launch():
        ctx.decode_step(batch=B, kv_len=kv_dev, page_table=table_dev, max_pages=max_pages, max_kv_len=int(kv_len.max()) + 1,
                        token_ids=tok1, x_out=x_out, logits=logits, next_token=nxt, stream=sD)

    decode_launch()
    sD.synchronize()
    ctx.check(sD)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=sD):
        decode_launch()

    def decode_once():
        with torch.cuda.stream(sD):
            graph.replay()

    # ---- finetune instance
    tok = wl.make_token_ids(w, (ft.micro_batch, ft.seq_len))
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

    class Finetune:
        """One call = one whole training step on the given stream, then a wait for it (a trainer reads the loss there;
        the wait also lets the pool take back the step's activations)."""
        T = ft.tokens
        t = 0

        def finetune_unit(self, st):
            self.t += 1
            with torch.cuda.stream(st):
                torch.index_select(embf, 0, tok_dev, out=acts[0])
            saved = []
            for l in range(L):
                saved.append(ctx.lora_fwd(l, acts[l], acts[l + 1], ft.micro_batch, ft.seq_len, stream=st))
            ctx.head_fwd_bwd(acts[L], tg_dev, loss, d0, stream=st)
            d, dn = d0, d1
            for l in range(L - 1, -1, -1):
                ctx.lora_bwd(l, d, dn, saved[l], dA[l], dB[l], stream=st)
                d, dn = dn, d
            for l in range(L):
                for p in A[l]:
                    hb.adamw_step(masters[l][p][0], moms[l][p][0], moms[l][p][1], dA[l][p], A[l][p], step=self.t, lr=1e-4,
                                  zero_grad=True, stream=st)
                    hb.adamw_step(masters[l][p][1], moms[l][p][2], moms[l][p][3], dB[l][p], Bm[l][p], step=self.t, lr=1e-4,
                                  zero_grad=True, stream=st)
            st.synchronize()

    hz = Finetune()

    # ---- solo references
    for _ in range(3):
        decode_once()
    sD.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(sD)
    for _ in range(20):
        decode_once()
    e1.record(sD)
    sD.synchronize()
    dec_solo_ms = e0.elapsed_time(e1) / 20
    hz.finetune_unit(sF)
    import time
    t0 = time.perf_counter()
    for _ in range(args.steps):
        hz.finetune_unit(sF)
    ft_solo_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ctx.check(sF)

    def summarise(r):
        tp = r["tpot"]
        return {"finetune_tokens_per_s": r["tokens_per_s"], "finetune_ms_per_step": r["ms_per_step"],
                "tpot_ms_p50": float(np.percentile(tp, 50)), "tpot_ms_p99": float(np.percentile(tp, 99)),
                "within_slo": float(np.mean(tp <= args.slo_ms)), "decode_steps": int(len(tp)),
                "decode_tokens_per_s": B * len(tp) / r["elapsed"]}

    import gc
    gc.collect()
    gc.freeze()                                     # a full collection over the set-up's objects stops the host for ~20 ms
    closed = colocate.run_colocated(hz, sD, sF, decode_once, args.steps, 1, None)
    ctx.check(sD)
    pace = args.pace_ms if args.pace_ms is not None else 0.6 * args.slo_ms
    paced = colocate.run_colocated(hz, sD, sF, decode_once, args.steps, 1, pace)
    ctx.check(sD)
    st = pool.stats()
    # algorithmic work per step: decode reads every weight once plus the cached K/V; the finetune step multiplies by
    # the frozen weights forward and backward (no weight gradients), plus attention (causal half), adapters, output layer
    dec_bytes = 2 * (L * m.layer_params + m.vocab * H) + int(sum(int(n) + 1 for n in kv_len)) * 2 * m.kv_row_bytes * L
    lora_flops = 0
    dims = dict(q=(H, m.n_q * m.head_dim), k=(H, m.n_kv * m.head_dim), v=(H, m.n_kv * m.head_dim), o=(m.n_q * m.head_dim, H),
                gate=(H, m.ffn), up=(H, m.ffn), down=(m.ffn, H))
    for p in lora.targets:
        lora_flops += 6 * T * lora.rank * sum(dims[p])
    attn = ft.micro_batch * 7 * ft.seq_len * ft.seq_len * m.n_q * m.head_dim      # forward 2 S^2 H, backward 2.5 x that
    ft_flops = L * (4 * T * m.layer_params + lora_flops + attn) + 4 * T * m.vocab * H

    def roof(summary, dec_ms_mean):
        return dict(summary,
                    finetune_TFLOPs=ft_flops / (summary["finetune_ms_per_step"] * 1e-3) / 1e12,
                    finetune_frac_of_2500_TFLOPs=ft_flops / (summary["finetune_ms_per_step"] * 1e-3) / 1e12 / 2500.0,
                    decode_GBs=dec_bytes / (dec_ms_mean * 1e-3) / 1e9, decode_frac_of_8000_GBs=dec_bytes / (dec_ms_mean * 1e-3) / 1e9 / 8000.0)

    out = {"workload": "config %d, %d layers + output layer: decode batch %d (cached tokens %d..%d) beside a finetune step of %d x %d "
                       "tokens, LoRA r=%d on %s" % (args.config, L, B, kv_len.min(), kv_len.max(), ft.micro_batch, ft.seq_len,
                                                    lora.rank, ",".join(lora.targets)),
           "slo_tpot_ms": args.slo_ms,
           "algorithmic": {"decode_GB_per_step": dec_bytes / 1e9, "finetune_TFLOP_per_step": ft_flops / 1e12},
           "solo": {"decode_tpot_ms": dec_solo_ms, "decode_GBs": dec_bytes / (dec_solo_ms * 1e-3) / 1e9,
                    "decode_frac_of_8000_GBs": dec_bytes / (dec_solo_ms * 1e-3) / 1e9 / 8000.0,
                    "finetune_ms_per_step": ft_solo_ms, "finetune_tokens_per_s": T / ft_solo_ms * 1e3,
                    "finetune_TFLOPs": ft_flops / (ft_solo_ms * 1e-3) / 1e12,
                    "finetune_frac_of_2500_TFLOPs": ft_flops / (ft_solo_ms * 1e-3) / 1e12 / 2500.0},
           "colocated_closed_loop": roof(summarise(closed), float(np.mean(closed["tpot"]))),
           "colocated_paced": dict(summarise(paced), decode_interval_ms=pace,
                                   finetune_TFLOPs=ft_flops / (paced["ms_per_step"] * 1e-3) / 1e12,
                                   finetune_frac_of_2500_TFLOPs=ft_flops / (paced["ms_per_step"] * 1e-3) / 1e12 / 2500.0),
           "pool": {"chunks": st.n_chunks, "kv_chunks": st.kv_chunks, "chunk_MB": chunk / 1e6, "slab_GB": slab_bytes / 1e9,
                    "library_GB_in_pool": ctx.device_bytes().in_pool / 1e9, "library_GB_outside_pool": ctx.device_bytes().outside_pool / 1e9},
           "loss_last": float(loss)}
    # let go of the device memory before the caller goes on
    del graph
    return out


if __name__ == "__main__":
    main()
