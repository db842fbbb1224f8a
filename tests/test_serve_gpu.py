"""A request trace served next to a finetune task on one unified pool (device): continuous batching allocates and frees
KV pages as sequences start, grow and finish, the finetune task takes its activations from the same pool and backs off
under pressure, and at the end every page and block is back in the pool.  The decode arithmetic itself is covered by
tests/test_decode_gpu.py; here the moving page tables are checked through a second, static run of the same sequence."""
import argparse
import dataclasses

import pytest
import torch

import workloads as wl
from paper_2511_11729_amd import bench_serve, serve

pytestmark = pytest.mark.gpu


def small(pool_gb=None, max_batch=12, max_len=200, ft_tokens=(2, 64)):
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16", n_layers=2, vocab=512)
    args = argparse.Namespace(config=0, layers=None, vocab=None, ft_tokens=ft_tokens, pool_gb=pool_gb, max_batch=max_batch,
                              max_len=max_len, release_ms=12.0, slo_ms=40.0)
    return (args,) + bench_serve.build(args, model=m)


def test_trace_with_finetune_beside_it_leaves_the_pool_clean():
    args, w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep = small()
    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()
    server = serve.DecodeServer(ctx, pool, m, max_batch=args.max_batch, max_len=args.max_len, stream=sD, slab=keep[0])
    arrivals = wl.make_arrivals(w, 400, targets=(2, 6, 12, 4), mean_out=24, prompt=("uniform", 5, 120))
    res = serve.replay(server, arrivals, lambda: serve.FinetuneWorker(pool, ft_step, sF, ft.tokens))
    server.drain()
    ctx.check(sD)
    assert res["admitted"] >= res["finished"]
    assert res["finished"] > 20 and res["batch_max"] >= 6
    assert res["preempted"] == 0                                   # the reserve kept decode supplied
    assert res["finetune"]["steps"] >= 1
    assert res["tpot_ms_p99"] < 40.0
    st = pool.stats()
    torch.cuda.synchronize()
    pool.alloc_pages(0)                                            # lets the pool collect frees whose events completed
    st = pool.stats()
    assert st.kv_pages_live == 0 and st.tensor_blocks_live == 0 and st.small_bytes_live == 0


def test_tight_pool_makes_the_finetune_task_wait_not_decode():
    """A slab with room for the KV cache but not for a whole step's activations on top of the reserve: the finetune
    task runs into out-of-memory or pressure and retries; decode is never pre-empted and still finishes its requests."""
    # chunk = 2 layers x 2 x 2 MiB = 8 MiB; one layer of a 4 x 512-token step saves ~16 MB (more than two chunks), so six
    # chunks minus the KV chunk and the reserve cannot hold both layers
    args, w, m, ft, pool, ctx, ft_step, (n_chunks, chunk, slab_bytes, reserve), keep = small(
        pool_gb=((256 << 20) + 6 * (8 << 20) + 4096) / 1e9, ft_tokens=(4, 512))
    assert n_chunks == 6
    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()
    server = serve.DecodeServer(ctx, pool, m, max_batch=args.max_batch, max_len=args.max_len, stream=sD, slab=keep[0])
    arrivals = wl.make_arrivals(w, 300, targets=(4, 12), mean_out=24, prompt=("uniform", 5, 120))
    res = serve.replay(server, arrivals, lambda: serve.FinetuneWorker(pool, ft_step, sF, ft.tokens))
    server.drain()
    ctx.check(sD)
    f = res["finetune"]
    assert f["oom_retries"] + f["pressure_backoffs"] > 0
    assert res["preempted"] == 0 and res["finished"] > 10
    torch.cuda.synchronize()
    pool.alloc_pages(0)
    st = pool.stats()
    assert st.kv_pages_live == 0 and st.tensor_blocks_live == 0


def test_moving_page_tables_give_the_same_tokens_as_a_static_run():
    """One sequence served alone: the tokens the server produces step after step (argmax fed back) equal those of
    direct harli_decode_step calls on a fixed page table holding the same cache contents."""
    args, w, m, ft, pool, ctx, ft_step, sizes, keep = small(max_batch=4, max_len=120)
    sD = torch.cuda.Stream()
    server = serve.DecodeServer(ctx, pool, m, max_batch=4, max_len=120, stream=sD, slab=keep[0])
    server.submit([(37, 30)])
    got = []
    for _ in range(30):
        r = server.step()
        assert r is not None
        r[0].synchronize()
        got.append(int(server.tok[0]))                              # after the swap `tok` holds the tokens just produced
    assert server.finished == 1 and not server.running
    # static replay: same zero-initialised prompt cache (the slab starts zeroed and freed pages are reused as they are,
    # so take fresh pages from a second pool-less run: allocate, then decode step by step with one table)
    ids = pool.alloc_pages((37 + 30 + 1 + 15) // 16)
    idx = torch.tensor(ids, dtype=torch.int64, device="cuda:0")
    server.kv_view[idx // server.ppb, :, idx % server.ppb, :] = 0        # the same all-zero prompt cache
    torch.cuda.synchronize()
    table = torch.full((1, server.max_pages), -1, dtype=torch.int32, device="cuda:0")
    table[0, : len(ids)] = torch.tensor(ids, dtype=torch.int32)
    # the server's pages were (37 zeros of prompt, then its own appended tokens); zero the fresh pages the same way
    tok = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    nxt = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    logits = torch.empty(1, m.vocab, device="cuda:0")
    x_out = torch.empty(1, m.hidden, device="cuda:0")
    want = []
    for t in range(30):
        kv = torch.tensor([37 + t], dtype=torch.int32, device="cuda:0")
        ctx.decode_step(batch=1, kv_len=kv, page_table=table, max_pages=server.max_pages, max_kv_len=38 + t, token_ids=tok,
                        x_out=x_out, logits=logits, next_token=nxt, stream=sD)
        sD.synchronize()
        want.append(int(nxt[0]))
        tok, nxt = nxt, tok
    pool.free_pages(ids)
    assert got == want


def test_scheduled_trace_places_both_tasks_on_partitions_and_calibrates():
    """The request trace under the runtime scheduler: predictor profiled on the whole (small) model, one decision per
    decode phase, decode and finetune units moved between compute-unit partitions, measured step times folded back
    into the predictor.  Checks the plumbing end to end: valid plans, finetune progress, factors inside their clip,
    a clean pool, and no stream or event left behind (the process goes on to run other tests)."""
    args, w, m, ft, pool, ctx, ft_step, info, keep = small(max_batch=32, max_len=600, ft_tokens=(4, 128))
    args.sched_margin, args.static, args.no_feedback, args.ft_all_cus = 0.9, None, False, False
    args.slo_ms = 5.0
    sD = torch.cuda.Stream()
    with torch.cuda.stream(sD):
        keep[-1].zero_()
    sD.synchronize()
    server = serve.DecodeServer(ctx, pool, m, max_batch=args.max_batch, max_len=args.max_len, stream=sD, slab=keep[0])
    plan, rep, cs = bench_serve.make_plan(args, m, ft, pool, ctx, ft_step, server, lambda *a: None)
    assert len(cs.shared_pipe) <= 4                                # partitions left on a shared dispatch pipe (normally none)
    assert rep["eq1_mean_abs_err_fitted_points"] < 0.5 and rep["eq2_b1_k1"][0] > 0
    arrivals = wl.make_arrivals(w, 300, targets=(2, 8, 24, 6), mean_out=24, prompt=("uniform", 5, 400))
    res = serve.replay(server, arrivals, lambda: serve.FinetuneWorker(pool, ft_step, None, ft.tokens), slo_ms=args.slo_ms, plan=plan)
    server.drain()
    server.use_stream(sD)
    ctx.check(sD)
    cs.close()
    plans = res["plans"]
    assert len(plans) == res["decode_steps"] > 100
    for i, f, act, pred_ms, n in plans:
        assert 1 <= i <= 10 and 0 <= f <= 10 - i
        assert f > 0 or i == 10                                    # paused or starved: inference has the whole chip
    assert res["finetune"]["steps"] >= 1 and res["preempted"] == 0
    assert res["within_slo"] >= 0.9, res["tpot_ms_p99"]
    assert all(0.6 <= s_ <= 2.5 for s_ in rep["calibration_by_level"][1:])
    assert any(abs(s_ - 1.0) > 1e-6 for s_ in rep["calibration_by_level"][1:])        # steps were timed and folded back
    torch.cuda.synchronize()
    pool.alloc_pages(0)
    st = pool.stats()
    assert st.kv_pages_live == 0 and st.tensor_blocks_live == 0
