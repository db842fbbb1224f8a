#!/usr/bin/env python3
"""Co-location benchmark of the Harli hot path on one MI355X.

Workload (config 1, synthetic): one 7B-class decoder layer (hidden 4096, 32 x 128 heads, SwiGLU
ffn 11008, bf16 weights).  Two tasks share the GPU and one unified memory pool, each on its own
HIP stream (the paper's two model instances in one process, Sec. 7):
  * decode  -- batch 8, cached lengths uniform in [256, 2048], 16-token pages; steps are issued
               back to back from a host thread for the whole timed window (closed loop);
  * finetune -- LoRA r=16 on q,k,v,o, micro-batch 4 x 512 tokens, layer forward + backward
               (the paper's per-layer scheduling unit, Sec. 6.1).
One "step" = one finetune unit (forward + backward of one micro-batch) with decode running
beside it.  Metric: finetune tokens/s while the decode time-per-output-token stays inside the
SLO (40 ms for a 32-layer model = 1.25 ms for this one layer).  `value` is the closed-loop case (decode
unthrottled, the hardest neighbour); `slo_paced` repeats the run with one decode step issued every 0.6 x SLO,
the operating point of a request stream that needs the SLO and no more.

Prints ONE JSON line.  `roofline` is the finetune unit's MFMA GEMM (the kernel that dominates the
step): algorithmic flops per launch over its event-timed duration, against the 2.5 PFLOP/s dense
16-bit MFMA peak.  `roofline_decode` is the decode step: algorithmic bytes per step (layer
weights + cached K/V read once) over the step time, against 8 TB/s.  `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same finetune workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SLO_MS_FULL_MODEL = 40.0          # paper Sec. 8.1: TPOT QoS target
PEAK_MFMA_TFLOPS = 2500.0         # MI355X dense fp16/bf16
PEAK_HBM_GBS = 8000.0
# HBM traffic per launch / per step from the rocprofv3 FETCH_SIZE and WRITE_SIZE counter runs summarised in
# profiles/bench_config1_hbm_traffic.md (each scaled by what the same counter reads for a 256 MiB device copy)
TRAFFIC_GEMM_BYTES_PER_LAUNCH = 377.1e6      # k_gemm, average over the 11 launches of a finetune unit
TRAFFIC_DECODE_BYTES_PER_STEP = 559.5e6      # all kernels of one decode step


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--solo", action="store_true", help="also report each task running alone (default on)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region run three plain 256 MiB device copies: the known-size kernel that the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the data-parallel path; --gpus %d is not supported "
              "(every rank would run this same single-GPU workload independently)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2511_11729_amd import binding as hb
    from tests.gpu_util import to_dev, f32_dev        # device upload helpers only (no arithmetic)

    hb.lib()                                          # fails loudly when libharli.so is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.workload(1)
    m, ft, lora = w.model, w.finetune, w.lora
    K, W = args.steps, args.warmup
    T = ft.tokens
    slo_ms = SLO_MS_FULL_MODEL / 32.0

    # ------------------------------------------------------------------ inputs (seeded, synthetic)
    log("[bench] generating config-1 weights and inputs")
    W_np = wl.make_layer_weights(w, 0)
    lora_np = wl.make_lora(w, 0)
    x_np, kv_len, kv_np = wl.make_decode_inputs(w)
    X_np, _ = wl.make_finetune_inputs(w)
    B = len(kv_len)
    P = 16
    n_pages = [(int(n) + 1 + P - 1) // P for n in kv_len]
    total_pages = sum(n_pages)

    # ------------------------------------------------------------------ one unified pool for KV pages and activations
    block = 2 << 20
    chunk = m.n_layers * 2 * block
    ppb = block // (P * m.kv_row_bytes)
    act_bytes_est = (T * m.hidden * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6
                     + ft.micro_batch * m.n_q * ft.seq_len * ft.seq_len * 2)
    in_flight = 8                                      # finetune micro-batches whose release events may be pending
    n_chunks = -(-total_pages // ppb) + in_flight * (act_bytes_est // chunk + 2) + 4
    small = 64 << 20
    slab_bytes = small + n_chunks * chunk
    slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=dev)
    pool = hb.Pool(slab, slab_bytes, block_bytes=block, n_layers=m.n_layers, kv_row_bytes=m.kv_row_bytes,
                   small_pool_bytes=small, kv_reserve_chunks=2)
    ids = np.array(pool.alloc_pages(total_pages), np.int64)[wl.page_order(w, total_pages)]
    max_pages = max(n_pages) + 1
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :n_pages[b]] = ids[k:k + n_pages[b]]
        k += n_pages[b]
    # KV contents: the values do not change the traffic; fill the pages with the seeded draws
    img = np.zeros(slab_bytes // 2, np.uint16)
    d = m.head_dim
    for b in range(B):
        Kc, Vc = kv_np[0][b]
        for which, Tn in ((0, Kc), (1, Vc)):
            enc = wl.bf16_bits(Tn).reshape(Tn.shape)
            n = Tn.shape[0]
            for lp in range((n + P - 1) // P):
                t0, t1 = lp * P, min(n, lp * P + P)
                base = pool.kv_addr(int(table[b, lp]), 0, which) // 2
                for c in range(m.n_kv):
                    off = base + c * P * d
                    img[off: off + (t1 - t0) * d] = enc[t0:t1, c, :].reshape(-1)
    slab.copy_(torch.from_numpy(img.view(np.uint8)))
    del img

    layer_dev = {n: to_dev(W_np[n], "bf16") for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
    layer_dev["g1"], layer_dev["g2"] = f32_dev(W_np["g1"]), f32_dev(W_np["g2"])
    ctx = hb.Context(pool, n_layers=1, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim,
                     ffn=m.ffn, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=B,
                     max_seq_len=int(kv_len.max()) + 8, max_ft_tokens=T, layers=[layer_dev])
    A_dev = {p: to_dev(a, "bf16") for p, (a, b) in lora_np.items()}
    B_dev = {p: to_dev(b, "bf16") for p, (a, b) in lora_np.items()}
    ctx.lora_attach(lora.rank, lora.alpha, lora.targets, [A_dev], [B_dev])

    kv_len_dev = torch.from_numpy(kv_len.astype(np.int32)).to(dev)
    table_dev = torch.from_numpy(table).to(dev)
    x_dev = f32_dev(x_np)
    y_dev = torch.empty(B, m.hidden, dtype=torch.float32, device=dev)
    X_dev = f32_dev(X_np.reshape(T, m.hidden))
    Y_dev = torch.empty(T, m.hidden, dtype=torch.float32, device=dev)
    dY_dev = torch.randn(T, m.hidden, dtype=torch.float32, device=dev, generator=torch.Generator(dev).manual_seed(1003)) / (T * m.hidden)
    dX_dev = torch.empty(T, m.hidden, dtype=torch.float32, device=dev)
    dA = {p: torch.zeros(a.shape, dtype=torch.float32, device=dev) for p, (a, b) in lora_np.items()}
    dB = {p: torch.zeros(b.shape, dtype=torch.float32, device=dev) for p, (a, b) in lora_np.items()}
    max_kv = int(kv_len.max()) + 1

    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()   # default priority on both

    def decode_launch():
        ctx.decode_step(batch=B, kv_len=kv_len_dev, page_table=table_dev, max_pages=max_pages, max_kv_len=max_kv,
                        x_in=x_dev, x_out=y_dev, stream=sD)

    ft_done = []                                       # one event per finished unit: bounds the units in flight

    def finetune_unit():
        if len(ft_done) >= in_flight - 2:
            ft_done[-(in_flight - 2)].synchronize()    # their pool memory is released by events, keep <= 6 pending
        sv = ctx.lora_fwd(0, X_dev, Y_dev, ft.micro_batch, ft.seq_len, stream=sF)
        ctx.lora_bwd(0, dY_dev, dX_dev, sv, dA, dB, stream=sF)
        ev = torch.cuda.Event()
        ev.record(sF)
        ft_done.append(ev)

    # decode step as one graph launch (no memset nodes inside); falls back to direct launches
    graph = None
    try:
        decode_launch()
        sD.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=sD):
            decode_launch()
        g.replay()
        sD.synchronize()
        graph = g
    except Exception as e:                             # pragma: no cover
        log("[bench] decode graph capture unavailable (%s); using direct launches" % e)
    ctx.check(sD)

    def decode_once():
        if graph is not None:
            with torch.cuda.stream(sD):
                graph.replay()
        else:
            decode_launch()

    kv_bytes = int(sum(int(n) + 1 for n in kv_len)) * 2 * m.kv_row_bytes
    dec_bytes = 2 * m.layer_params + kv_bytes

    # ------------------------------------------------------------------ solo references
    def time_decode_solo(n=300):
        for _ in range(20):
            decode_once()
        sD.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(sD)
        for _ in range(n):
            decode_once()
        e1.record(sD)
        sD.synchronize()
        return e0.elapsed_time(e1) / n

    def time_finetune_solo(n):
        for _ in range(2):
            finetune_unit()
        sF.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(sF)
        for _ in range(n):
            finetune_unit()
        e1.record(sF)
        sF.synchronize()
        return e0.elapsed_time(e1) / n

    log("[bench] solo runs")
    dec_solo_ms = time_decode_solo()
    ft_solo_ms = time_finetune_solo(max(3, min(K, 10)))
    pool.stats()                                       # polls release events

    # ------------------------------------------------------------------ co-located, timed
    def run_colocated(pace_ms):
        """K timed finetune units with decode beside them.  pace_ms None: decode steps back to back (closed loop);
        otherwise one decode step is issued every pace_ms (a request stream that only needs the SLO)."""
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
                    dec_end[i - 256].synchronize()     # bound the run-ahead of the host thread
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
        for _ in range(W):
            finetune_unit()
        sF.synchronize()
        torch.cuda.synchronize()
        hb.prof_enable(True)
        i0 = len(dec_end)
        t0 = time.perf_counter()
        for _ in range(K):
            finetune_unit()
        sF.synchronize()
        t1 = time.perf_counter()
        i1 = len(dec_end)
        stop.set()
        th.join()
        torch.cuda.synchronize()
        hb.prof_enable(False)
        gemm_flops, gemm_ms, gemm_n = hb.prof_collect()
        ctx.check(sD)
        elapsed = t1 - t0
        # time per output token: completion-to-completion interval of consecutive decode steps inside the window;
        # step latency: first kernel start to last kernel end of one step
        lo, hi = max(i0, 1) - 1, i1
        tpot = np.array([dec_end[j].elapsed_time(dec_end[j + 1]) for j in range(lo, hi - 1)]) if hi - lo > 2 else np.array([float("nan")])
        steplat = np.array([dec_start[j].elapsed_time(dec_end[j]) for j in range(lo, hi)]) if hi > lo else np.array([float("nan")])
        return {"elapsed": elapsed, "tokens_per_s": K * T / elapsed, "ms_per_step": elapsed * 1e3 / K,
                "tpot": tpot, "steplat": steplat, "gemm": (gemm_flops, gemm_ms, gemm_n)}

    log("[bench] co-located, decode in a closed loop: %d warmup + %d timed finetune units" % (W, K))
    closed = run_colocated(None)
    pace_ms = 0.6 * slo_ms
    log("[bench] co-located, one decode step every %.2f ms (0.6 x SLO)" % pace_ms)
    paced = run_colocated(pace_ms)
    elapsed, ms_per_step, tokens_per_s = closed["elapsed"], closed["ms_per_step"], closed["tokens_per_s"]
    gemm_flops, gemm_ms, gemm_n = closed["gemm"]
    lat = closed["tpot"]
    tpot_p50, tpot_p99, tpot_mean = float(np.percentile(lat, 50)), float(np.percentile(lat, 99)), float(lat.mean())

    # ------------------------------------------------------------------ CPU baseline: the oracle on a bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import harli_oracle as O
        sb, ss = 4, 512                                # the whole micro-batch, full layer width (about 10-20 s)
        log("[bench] CPU oracle baseline on %d x %d tokens" % (sb, ss))
        sh = O.Shapes(m.hidden, m.n_q, m.n_kv, m.head_dim, m.ffn, m.rms_eps, m.rope_base)
        Xs = X_np[:sb, :ss]
        reps = 0
        c0 = time.perf_counter()
        while True:                                    # whole micro-batches until about 12 s of CPU work
            Yo, sv = O.layer_forward(Xs, W_np, lora_np, lora.scale, sh)
            _, dYo = O.mse_loss(Yo, np.zeros_like(Yo))
            O.layer_backward(dYo, sv, W_np, lora_np, lora.scale, sh)
            reps += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 12.0 or reps >= 16:
                break
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        cpu = {"value": reps * sb * ss / (c1 - c0), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": "numpy fp64 layer forward+backward of the %d x %d micro-batch at full 7B-layer width, repeated "
                         "%d times (%.1f s), decode not running" % (sb, ss, reps, c1 - c0)}

    if args.calib_copy:
        src = torch.full((64 << 20,), 1.0, dtype=torch.float32, device=dev)     # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # measured ceilings of this GPU (plain read kernels of the library's debug ABI): what HBM and the L2 caches deliver
    probe = torch.empty(6 << 30, dtype=torch.uint8, device=dev)
    peaks = {"hbm_stream_read_GBs": hb.dbg_read_bandwidth(probe, 0), "l2_to_cu_read_GBs": hb.dbg_read_bandwidth(probe, 1),
             "note": "the GEMM's workgroups pull (256+128) x K x 2 bytes of operand panels per 256x128 tile through L2: at "
                     "the L2 rate above that bounds it below the MFMA peak"}
    del probe

    ach_tf = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else float("nan")
    out = {
        "metric": "LoRA finetune tokens/s under decode TPOT SLO",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 MFMA operands / fp32 accumulate (finetune); bf16 / fp32 (decode)", "data": "synthetic",
        "config": {"workload": "config 1: one 7B-class decoder layer; decode batch 8, KV lengths U[256,2048], 16-token "
                               "pages, closed loop on stream D; LoRA r=16 q,k,v,o finetune, micro-batch 4x512, "
                               "forward+backward on stream F; one unified pool",
                   "finetune_tokens_per_step": T, "decode_batch": B, "slo_tpot_ms": slo_ms},
        "slo": {"tpot_ms_p50": tpot_p50, "tpot_ms_p99": tpot_p99, "tpot_ms_mean": tpot_mean, "limit_ms": slo_ms,
                "met": bool(tpot_p99 <= slo_ms), "decode_steps_in_window": int(len(lat)),
                "decode_step_latency_ms_p50": float(np.percentile(closed["steplat"], 50)),
                "decode_step_latency_ms_p99": float(np.percentile(closed["steplat"], 99))},
        "roofline": {"bound": "mfma", "achieved": ach_tf, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach_tf / PEAK_MFMA_TFLOPS, "traffic": TRAFFIC_GEMM_BYTES_PER_LAUNCH, "kernel": "k_gemm<half>",
                     "launches": int(gemm_n), "avg_launch_us": gemm_ms * 1e3 / max(gemm_n, 1),
                     "note": "co-located with decode; flops = 2MNK per launch (causal launches count half)"},
        "roofline_decode": {"bound": "hbm", "achieved": dec_bytes / (tpot_mean * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                            "unit": "GB/s", "frac": dec_bytes / (tpot_mean * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": TRAFFIC_DECODE_BYTES_PER_STEP,
                            "bytes_per_step": dec_bytes, "solo_achieved": dec_bytes / (dec_solo_ms * 1e-3) / 1e9,
                            "solo_frac": dec_bytes / (dec_solo_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "slo_paced": {"decode_interval_ms": pace_ms, "value": paced["tokens_per_s"], "unit": "tokens/s",
                      "ms_per_step": paced["ms_per_step"],
                      "tpot_ms_p50": float(np.percentile(paced["tpot"], 50)), "tpot_ms_p99": float(np.percentile(paced["tpot"], 99)),
                      "decode_step_latency_ms_p50": float(np.percentile(paced["steplat"], 50)),
                      "decode_step_latency_ms_p99": float(np.percentile(paced["steplat"], 99)),
                      "met": bool(np.percentile(paced["tpot"], 99) <= slo_ms),
                      "note": "same co-location with decode steps issued every 0.6 x SLO instead of back to back"},
        "solo": {"decode_ms_per_step": dec_solo_ms, "finetune_ms_per_step": ft_solo_ms,
                 "finetune_tokens_per_s": T / ft_solo_ms * 1e3},
        "measured_peaks": peaks,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
