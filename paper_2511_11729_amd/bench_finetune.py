"""Finetune-only timing of a full model on one GPU:  python -m paper_2511_11729_amd.bench_finetune --config 2

One step = embedding gather, every layer's LoRA forward, the output layer with next-token cross entropy, every
layer's backward (the paper's per-layer units, Sec. 6.1, chained through explicit hand-off tensors) and an AdamW
update of every adapter.  Seeded random weights; every layer shares ONE set of host-generated frozen weights (the
library still keeps its own half-precision copies per layer), adapters are per layer.  Prints one JSON line with
tokens/s and the achieved rate on the algorithmic flops (4 T P_layer per layer for the base GEMMs, 4 T V H for the
output layer, causal attention and LoRA terms added).  --window n runs the step under a window of n device slots over
the frozen weights (the rest stays in pinned host memory and is copied in ahead of use) and reports the host-to-device
rate the step sustained.
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
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--window", type=int, default=0,
                    help="keep only this many layer copies of the frozen weights on the device (0: all resident)")
    args = ap.parse_args()

    import dataclasses
    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb
    from paper_2511_11729_amd.harness import dev_bf16, dev_f32

    hb.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.workload(args.config)
    m = w.model if args.layers is None else dataclasses.replace(w.model, n_layers=args.layers)
    if m.dtype != "bf16" or m.vocab <= 0:
        raise SystemExit("bench_finetune: needs a bf16 workload with an output layer (configs 2-4)")
    ft, lora = w.finetune, w.lora
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
    B = [{p: dev_bf16(b) for p, (a, b) in lora_np.items()} for _ in range(L)]

    block = 2 << 20
    chunk = L * 2 * block
    per_layer = T * H * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6
    n_chunks = (L + 1) * (per_layer // chunk + 2) + 4       # a unit's activations take whole adjacent chunks
    slot_chunks = -(-2 * m.layer_params // chunk) + 1        # one window slot: a layer's weights in one orientation
    n_chunks += min(args.window, 2 * L) * slot_chunks
    small = 256 << 20
    slab_bytes = small + n_chunks * chunk
    slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=dev)
    pool = hb.Pool(slab, slab_bytes, block_bytes=block, n_layers=L, kv_row_bytes=m.kv_row_bytes, small_pool_bytes=small,
                   kv_reserve_chunks=1)
    ctx = hb.Context(pool, n_layers=L, hidden=H, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim, ffn=m.ffn,
                     vocab=m.vocab, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=1, max_seq_len=16,
                     max_ft_tokens=T, layers=[layer] * L, emb=emb, g_final=gf, w_lm=wlm)
    ctx.lora_attach(lora.rank, lora.alpha, lora.targets, A, B)
    if args.window > 0:
        ctx.ft_window_enable(args.window)

    tok = wl.make_token_ids(w, (ft.micro_batch, ft.seq_len))
    tg = np.full(tok.shape, -1, np.int32)
    tg[:, :-1] = tok[:, 1:]
    tok_dev = torch.from_numpy(tok.reshape(-1).astype(np.int64)).to(dev)
    tg_dev = torch.from_numpy(tg.reshape(-1)).to(dev)
    acts = [torch.empty(T, H, dtype=torch.float32, device=dev) for _ in range(L + 1)]
    d0, d1 = torch.empty(T, H, device=dev), torch.empty(T, H, device=dev)
    loss = torch.zeros(1, device=dev)
    masters = [{p: (A[l][p].float(), B[l][p].float()) for p in A[l]} for l in range(L)]
    moms = [{p: [torch.zeros_like(masters[l][p][0]), torch.zeros_like(masters[l][p][0]), torch.zeros_like(masters[l][p][1]),
                 torch.zeros_like(masters[l][p][1])] for p in A[l]} for l in range(L)]
    dA = [{p: torch.zeros_like(masters[l][p][0]) for p in A[l]} for l in range(L)]
    dB = [{p: torch.zeros_like(masters[l][p][1]) for p in A[l]} for l in range(L)]
    st = torch.cuda.Stream()
    embf = emb.float()                                   # gather source (harness side)

    def step(t):
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
                hb.adamw_step(masters[l][p][0], moms[l][p][0], moms[l][p][1], dA[l][p], A[l][p], step=t, lr=1e-4, zero_grad=True, stream=st)
                hb.adamw_step(masters[l][p][1], moms[l][p][2], moms[l][p][3], dB[l][p], B[l][p], step=t, lr=1e-4, zero_grad=True, stream=st)

    step(1)
    st.synchronize()
    ctx.check(st)
    l0 = float(loss)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    h2d0 = ctx.ft_window_stats().h2d_bytes
    e0.record(st)
    for t in range(args.steps):
        step(t + 2)
        st.synchronize()          # a trainer reads the loss here; it also lets the pool take back the step's activations
    e1.record(st)
    st.synchronize()
    ctx.check(st)
    ms = e0.elapsed_time(e1) / args.steps
    ws = ctx.ft_window_stats()
    window = None
    if ws.slots > 0:
        per_step = (ws.h2d_bytes - h2d0) / args.steps       # what the timed steps copied from the host
        window = {"slots": ws.slots, "slot_MB": ws.slot_bytes / 1e6, "host_pinned_GB": ws.host_bytes / 1e9,
                  "h2d_GB_per_step": per_step / 1e9, "h2d_GBs": per_step / ms / 1e6, "hits": ws.hits, "misses": ws.misses,
                  "refills": ws.refills}
    r = lora.rank
    lora_flops = 0
    for p in lora.targets:
        o, i = m.proj_shape(p)
        lora_flops += 6 * T * r * (i + o)                # forward 2, backward 4 (dx and the two gradients)
    attn = 3.5 * 2 * ft.seq_len * ft.seq_len * H * ft.micro_batch     # causal forward 2 S^2 H per sequence, backward 2.5x
    flops = L * (4 * T * m.layer_params + lora_flops + attn) + 4 * T * m.vocab * H
    print(json.dumps({"workload": "config %d finetune, %d layers + output layer, micro-batch %d x %d, LoRA r=%d on %s" %
                                  (args.config, L, ft.micro_batch, ft.seq_len, r, ",".join(lora.targets)),
                      "ms_per_step": ms, "tokens_per_s": T / ms * 1e3, "algorithmic_TFLOP_per_step": flops / 1e12,
                      "achieved_TFLOPs": flops / ms / 1e9, "frac_of_2.5PF": flops / ms / 1e9 / 2500.0,
                      "loss_first": l0, "loss_last": float(loss), "steps": args.steps, "window": window}))


if __name__ == "__main__":
    main()
