"""Decode-only timing of a full model on one GPU:  python -m paper_2511_11729_amd.bench_decode --config 2 --batch 16

Builds the named workload's model at full depth with seeded random weights (every layer shares ONE set of
host-generated layer weights -- the traffic is the same, the library still keeps a private pre-shuffled copy per
layer), fills the paged KV cache with zeros at the workload's cached lengths, captures one decode step
(embedding, all layers, output layer, argmax) in a HIP graph and replays it.  Prints one JSON line with the time
per output token, the algorithmic bytes per step (layer weights + output layer + cached K/V, each read once) and
the achieved fraction of 8 TB/s.
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
    ap.add_argument("--batch", type=int, default=None, help="decode batch (default: the workload's)")
    ap.add_argument("--kv-len", type=int, default=None, help="cached tokens per sequence (default: the workload's draw)")
    ap.add_argument("--layers", type=int, default=None, help="depth override")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--large-min-batch", type=int, default=0, help="measurement hook: smallest batch that runs the tiled GEMMs (0: the library's own)")
    args = ap.parse_args()
    print(json.dumps(run(args)))


def run(args):
    """The measurement itself; `args` carries config, batch, kv_len, layers, steps, large_min_batch.  Returns the result
    dictionary (bench.py calls this for its large-batch decode leg)."""
    import dataclasses
    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb

    hb.lib()
    if args.large_min_batch:
        hb.dbg_decode_large_min_batch(args.large_min_batch)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.workload(args.config)
    m = w.model if args.layers is None else dataclasses.replace(w.model, n_layers=args.layers)
    if m.dtype != "bf16" or m.vocab <= 0:
        raise SystemExit("bench_decode: needs a bf16 workload with an output layer (configs 2-4)")
    B = args.batch or w.decode.batch
    kv_len = (np.full(B, args.kv_len, np.int32) if args.kv_len is not None else wl.draw_lengths(w, B)).astype(np.int32)
    P, L = 16, m.n_layers

    def dev_bf16(a):
        return torch.from_numpy(wl.bf16_bits(a).view(np.int16).reshape(a.shape)).to(dev).view(torch.bfloat16)

    def dev_f32(a):
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)

    W_np = wl.make_layer_weights(w, 0, m)
    ex = wl.make_model_extras(w, m)
    layer = {n: dev_bf16(W_np[n]) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
    layer["g1"], layer["g2"] = dev_f32(W_np["g1"]), dev_f32(W_np["g2"])
    for bn in ("bq", "bk", "bv"):
        if bn in W_np:
            layer[bn] = dev_f32(W_np[bn])
    emb, gf, wlm = dev_bf16(ex["emb"]), dev_f32(ex["gf"]), dev_bf16(ex["wlm"])

    block = 2 << 20
    chunk = L * 2 * block
    ppb = block // (P * m.kv_row_bytes)
    n_pages = [(int(n) + 1 + P - 1) // P for n in kv_len]
    total_pages = sum(n_pages)
    n_chunks = -(-total_pages // ppb) + 1
    slab_bytes = n_chunks * chunk
    slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=dev)
    pool = hb.Pool(slab, slab_bytes, block_bytes=block, n_layers=L, kv_row_bytes=m.kv_row_bytes, small_pool_bytes=0,
                   kv_reserve_chunks=0)
    ids = np.array(pool.alloc_pages(total_pages), np.int64)[wl.page_order(w, total_pages)]
    max_pages = max(n_pages) + 1
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :n_pages[b]] = ids[k:k + n_pages[b]]
        k += n_pages[b]
    ctx = hb.Context(pool, n_layers=L, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim, ffn=m.ffn,
                     rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=B,
                     max_seq_len=int(kv_len.max()) + 8, layers=[layer] * L, emb=emb, g_final=gf, w_lm=wlm, vocab=m.vocab)
    kv_dev = torch.from_numpy(kv_len).to(dev)
    table_dev = torch.from_numpy(table).to(dev)
    tok = torch.from_numpy(wl.make_token_ids(w, (B,)).astype(np.int32)).to(dev)
    x_out = torch.empty(B, m.hidden, dtype=torch.float32, device=dev)
    logits = torch.empty(B, m.vocab, dtype=torch.float32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    st = torch.cuda.Stream()

    def step():
        ctx.decode_step(batch=B, kv_len=kv_dev, page_table=table_dev, max_pages=max_pages, max_kv_len=int(kv_len.max()) + 1,
                        token_ids=tok, x_out=x_out, logits=logits, next_token=nxt, stream=st)

    step()
    st.synchronize()
    ctx.check(st)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        step()
    with torch.cuda.stream(st):
        for _ in range(3):
            g.replay()
        st.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            g.replay()
        e1.record(st)
        st.synchronize()
    ctx.check(st)
    ms = e0.elapsed_time(e1) / args.steps
    kv_bytes = int(sum(int(n) + 1 for n in kv_len)) * 2 * m.kv_row_bytes * L
    w_bytes = 2 * (L * m.layer_params + m.vocab * m.hidden)
    total = w_bytes + kv_bytes
    return {"workload": "config %d decode, %d layers, batch %d, cached tokens %d..%d" % (args.config, L, B, kv_len.min(), kv_len.max()),
            "tpot_ms": ms, "tokens_per_s": B / ms * 1e3, "bytes_per_step": total, "weight_bytes": w_bytes,
            "kv_bytes": kv_bytes, "achieved_GBs": total / ms / 1e6, "frac_of_8TBs": total / ms / 1e6 / 8000.0,
            "steps": args.steps}


if __name__ == "__main__":
    main()
