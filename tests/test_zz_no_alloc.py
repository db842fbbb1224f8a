"""harli_decode_step_static (the decode step on the library's static scratch array, for callers that cannot
allocate) against harli_decode_step through the C ABI: same kernels on the same inputs, so the same bits -- hidden
state, logits, chosen tokens and every byte of the KV slab -- on two calls in a row, the second with a smaller input
that finds the first one's leftovers in the array."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import DEV, DecodeCase, assert_close

pytestmark = pytest.mark.gpu


def both_ways(case, tok):
    """One step through each entry point from the same slab image; returns the two result sets."""
    out = []
    for static in (False, True):
        case.slab.copy_(torch.from_numpy(case.img0.view(np.uint8)))
        B, m = case.B, case.m
        y = torch.full((B, m.hidden), float("nan"), dtype=torch.float32, device=DEV)
        logits = torch.full((B, m.vocab), float("nan"), dtype=torch.float32, device=DEV)
        nxt = torch.full((B,), -1, dtype=torch.int32, device=DEV)
        step = case.ctx.decode_step_static if static else case.ctx.decode_step
        step(batch=B, kv_len=case.kv_len_dev, page_table=case.table_dev, max_pages=case.max_pages,
             max_kv_len=int(case.kv_len.max()) + 1, token_ids=torch.from_numpy(tok).to(DEV), logits=logits,
             next_token=nxt, x_out=y)
        torch.cuda.synchronize()
        case.ctx.check()
        out.append((y, logits, nxt, case.slab.clone()))
    return out


def test_static_scratch_step_equals_the_allocating_step_twice_in_a_row():
    w = wl.workload(0)
    # ffn 688 is not a multiple of 32: the contraction padding of the down projection's operand must be zero
    m = dataclasses.replace(w.model, dtype="bf16", n_layers=3, vocab=1000)
    wm = dataclasses.replace(w, model=m)
    big = DecodeCase(w, m, np.asarray([12, 200, 0, 77, 300, 33, 5, 129, 64, 511, 17, 256, 90, 1, 640, 31, 100], np.int32),
                     full_model=True, block_bytes=64 << 10)
    small = DecodeCase(w, m, np.asarray([40, 3, 130], np.int32), full_model=True, block_bytes=64 << 10)
    for case in (big, small):                       # the second call is smaller and lays the array out differently
        tok = wl.make_token_ids(wm, (case.B,))
        need = case.ctx.decode_step_static_bytes(case.B, int(case.kv_len.max()) + 1)
        assert 0 < need <= 64 << 20
        (y0, l0, n0, s0), (y1, l1, n1, s1) = both_ways(case, tok)
        assert torch.equal(y0, y1) and torch.equal(l0, l1) and torch.equal(n0, n1) and torch.equal(s0, s1)
        ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
        assert_close(y1.cpu().numpy(), ref_hid, "hidden state on the static scratch")
        assert_close(l1.cpu().numpy(), ref_logits, "logits on the static scratch")


def test_static_scratch_step_at_100_sequences_meets_the_oracle():
    """Above 32 sequences harli_decode_step runs its GEMMs tiled, with partial tiles in a workspace of its context; the
    static array has no room for that, so this entry point keeps the pass-wise kernels there.  Different summation
    orders, hence the comparison at the parity bar instead of bit for bit."""
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16", n_layers=2, vocab=1000)
    wm = dataclasses.replace(w, model=m)
    case = DecodeCase(w, m, np.asarray([5 + (i * 13) % 120 for i in range(100)], np.int32), full_model=True, block_bytes=64 << 10)
    tok = wl.make_token_ids(wm, (case.B,))
    assert 0 < case.ctx.decode_step_static_bytes(case.B, int(case.kv_len.max()) + 1) <= 64 << 20
    (y0, l0, n0, s0), (y1, l1, n1, s1) = both_ways(case, tok)
    ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
    for y, l, what in ((y0, l0, "allocating step"), (y1, l1, "static scratch")):
        assert_close(y.cpu().numpy(), ref_hid, "hidden state, " + what)
        assert_close(l.cpu().numpy(), ref_logits, "logits, " + what)


def test_static_scratch_step_refuses_what_does_not_fit():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    case = DecodeCase(w, m, np.asarray([5, 20], np.int32), block_bytes=64 << 10)
    layers = case.layers_dev
    big_ctx = hb.Context(case.pool, n_layers=m.n_layers, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv,
                         head_dim=m.head_dim, ffn=m.ffn, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16,
                         max_batch=64, max_seq_len=200000, layers=layers)
    assert big_ctx.decode_step_static_bytes(64, 150000) > 64 << 20
    x = torch.zeros(64, m.hidden, dtype=torch.float32, device=DEV)
    y = torch.empty_like(x)
    lens = torch.zeros(64, dtype=torch.int32, device=DEV)
    table = torch.zeros(64, 1, dtype=torch.int32, device=DEV)   # never read: the call is refused on the host
    with pytest.raises(hb.HarliError) as e:
        big_ctx.decode_step_static(batch=64, kv_len=lens, page_table=table, max_pages=10000, max_kv_len=150000, x_in=x, x_out=y)
    assert e.value.status == hb.HARLI_ERR_INVALID and "static buffer" in str(e.value)
    # fp32 storage is refused too
    m32 = w.model
    c32 = DecodeCase(w, m32, np.asarray([5], np.int32), block_bytes=64 << 10)
    with pytest.raises(hb.HarliError) as e:
        c32.ctx.decode_step_static(batch=1, kv_len=c32.kv_len_dev, page_table=c32.table_dev, max_pages=c32.max_pages,
                                   max_kv_len=6, x_in=c32.x_dev, x_out=torch.empty(1, m32.hidden, device=DEV))
    assert e.value.status == hb.HARLI_ERR_INVALID
    # and the step that fits still runs
    torch.cuda.synchronize()
    case.ctx.check()
