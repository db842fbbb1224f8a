"""Error behaviour of the compute entry points, through the C ABI on a device.

Every rejection below is decided on the host before anything is enqueued: the call returns its status, the pool and
the slab are untouched, and the next valid call gives the oracle's result.
"""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import DEV, DecodeCase, FinetuneCase, assert_close

pytestmark = pytest.mark.gpu


def rejected(status, fn, *a, **kw):
    with pytest.raises(hb.HarliError) as e:
        fn(*a, **kw)
    assert e.value.status == status, str(e.value)


def test_decode_step_rejects_what_its_header_says_and_enqueues_nothing():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    case = DecodeCase(w, m, np.asarray([5, 20, 33], np.int32), block_bytes=64 << 10, max_batch=4)
    B, H = case.B, m.hidden
    y = torch.empty(B, H, dtype=torch.float32, device=DEV)
    tok = torch.zeros(B, dtype=torch.int32, device=DEV)
    logits = torch.empty(B, 8, dtype=torch.float32, device=DEV)
    nxt = torch.empty(B, dtype=torch.int32, device=DEV)
    good = dict(batch=B, kv_len=case.kv_len_dev, page_table=case.table_dev, max_pages=case.max_pages,
                max_kv_len=int(case.kv_len.max()) + 1, x_in=case.x_dev, x_out=y)
    step = case.ctx.decode_step
    inv = hb.HARLI_ERR_INVALID
    rejected(inv, step, **dict(good, batch=0))
    rejected(inv, step, **dict(good, batch=5))                               # above max_batch = 4
    rejected(inv, step, **dict(good, max_kv_len=0))
    rejected(inv, step, **dict(good, max_kv_len=int(case.kv_len.max()) + 9))  # beyond the context's max_seq_len
    rejected(inv, step, **dict(good, max_pages=2))                           # rows of 2 pages cannot hold 34 tokens
    rejected(inv, step, **dict(good, kv_len=None))
    rejected(inv, step, **dict(good, page_table=None))
    rejected(inv, step, **dict(good, x_in=None))                             # neither token ids nor activations
    rejected(inv, step, **dict(good, x_in=None, token_ids=tok))              # the context has no embedding table
    rejected(inv, step, **dict(good, logits=logits))                         # ... and no output layer
    rejected(inv, step, **dict(good, next_token=nxt))                        # a token choice needs logits
    torch.cuda.synchronize()
    case.ctx.check()
    assert np.array_equal(case.slab_image(), case.img0)                     # no token was appended, nothing was written
    assert_close(case.run_gpu(), case.run_oracle(), "decode output after the rejected calls")


def test_device_side_checks_report_through_ctx_check_and_every_kernel_exits_normally():
    """What only the device can see -- a page id outside the pool, a token id outside the vocabulary, a sequence
    longer than the bound the step was sized for -- sets a flag instead of being dereferenced; harli_ctx_check
    reports and clears it, and the next valid step gives the oracle's result."""
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16", n_layers=2, vocab=500)
    lengths = np.asarray([300, 20, 33], np.int32)
    case = DecodeCase(w, m, lengths, full_model=True, block_bytes=64 << 10)
    B = case.B
    tok = wl.make_token_ids(dataclasses.replace(w, model=m), (B,))
    y = torch.empty(B, m.hidden, dtype=torch.float32, device=DEV)
    logits = torch.empty(B, m.vocab, dtype=torch.float32, device=DEV)
    tok_dev = torch.from_numpy(tok).to(DEV)
    good = dict(batch=B, kv_len=case.kv_len_dev, page_table=case.table_dev, max_pages=case.max_pages,
                max_kv_len=int(lengths.max()) + 1, token_ids=tok_dev, logits=logits, x_out=y)

    def flagged(word, **kw):
        case.slab.copy_(torch.from_numpy(case.img0.view(np.uint8)))
        case.ctx.decode_step(**dict(good, **kw))
        torch.cuda.synchronize()
        with pytest.raises(hb.HarliError) as e:
            case.ctx.check()
        assert e.value.status == hb.HARLI_ERR_INVALID and word in str(e.value), str(e.value)
        case.ctx.check()                                                     # reported once, then clear

    n_pages = case.geom.n_chunks * case.geom.pages_per_block                 # ids run 0..n_pages-1
    bad_table = case.table_dev.clone()
    bad_table[1, 0] = n_pages + 7                                            # a page the attention of sequence 1 reads
    flagged("page id", page_table=bad_table)
    bad_table = case.table_dev.clone()
    bad_table[2, int(lengths[2]) // 16] = -1                                 # the page the new token of sequence 2 goes to
    flagged("page id", page_table=bad_table)
    bad_tok = tok_dev.clone()
    bad_tok[0] = m.vocab
    flagged("token", token_ids=bad_tok)
    flagged("longer than max_kv_len", max_kv_len=256)                        # sequence 0 holds 301 tokens
    # nothing sticks: the valid step is the oracle's
    case.slab.copy_(torch.from_numpy(case.img0.view(np.uint8)))
    hid = case.run_gpu(token_ids=tok)
    ref_hid, ref_logits, _ = case.run_oracle(token_ids=tok)
    assert_close(hid, ref_hid, "hidden state after the flagged steps")
    assert_close(case.logits_dev.cpu().numpy(), ref_logits, "logits after the flagged steps")
    case.check_cache()


def test_finetune_entry_points_reject_bad_arguments_and_keep_the_pool_clean():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    fc = FinetuneCase(w, m, w.lora, w.finetune)
    ft, T, H = fc.ft, fc.ft.tokens, m.hidden
    Y = torch.empty(T, H, dtype=torch.float32, device=DEV)
    inv, state = hb.HARLI_ERR_INVALID, hb.HARLI_ERR_STATE
    live0 = fc.pool.stats().tensor_blocks_live
    rejected(inv, fc.ctx.lora_fwd, 1, fc.X_dev, Y, ft.micro_batch, ft.seq_len)          # one layer only
    rejected(inv, fc.ctx.lora_fwd, -1, fc.X_dev, Y, ft.micro_batch, ft.seq_len)
    rejected(inv, fc.ctx.lora_fwd, 0, fc.X_dev, Y, ft.micro_batch + 1, ft.seq_len)      # more than max_ft_tokens
    rejected(inv, fc.ctx.lora_fwd, 0, fc.X_dev, Y, 1, 12)                               # sequence length not a multiple of 8
    rejected(inv, fc.ctx.lora_fwd, 0, None, Y, ft.micro_batch, ft.seq_len)
    rejected(inv, fc.ctx.lora_fwd, 0, fc.X_dev, None, ft.micro_batch, ft.seq_len)
    assert fc.pool.stats().tensor_blocks_live == live0                                  # nothing was reserved
    # the context has no output layer
    loss = torch.zeros(1, device=DEV)
    tg = torch.zeros(T, dtype=torch.int32, device=DEV)
    rejected(state, fc.ctx.head_fwd_bwd, fc.X_dev, tg, loss, torch.empty_like(fc.X_dev))
    # backward: a null record, null buffers
    fc.forward_gpu()
    dY = torch.zeros(T, H, dtype=torch.float32, device=DEV)
    dX = torch.empty_like(dY)
    dA = {p: torch.zeros(a.shape, dtype=torch.float32, device=DEV) for p, (a, b) in fc.lora_np.items()}
    dB = {p: torch.zeros(b.shape, dtype=torch.float32, device=DEV) for p, (a, b) in fc.lora_np.items()}
    rejected(inv, fc.ctx.lora_bwd, 0, dY, dX, None, dA, dB)
    rejected(inv, fc.ctx.lora_bwd, 0, None, dX, fc.saved, dA, dB)
    some = next(iter(dA))
    rejected(inv, fc.ctx.lora_bwd, 0, dY, dX, fc.saved, {p: t for p, t in dA.items() if p != some}, dB)
    # the record survived the rejected calls: the real backward pass still matches the oracle
    _, _, dY_ref, dX_ref, _ = fc.oracle()
    dXg, _ = fc.backward_gpu(dY_ref)
    assert_close(dXg, dX_ref, "dX after the rejected calls")
    # a context made without finetune capacity refuses adapters, and without adapters refuses the unit
    dc = DecodeCase(w, m, np.asarray([5], np.int32), block_bytes=64 << 10)
    rejected(state, dc.ctx.lora_fwd, 0, fc.X_dev, Y, 1, 8)
    rejected(state, dc.ctx.lora_attach, w.lora.rank, w.lora.alpha, w.lora.targets, [fc.A_dev], [fc.B_dev])


def test_adamw_step_rejects_bad_hyperparameters_and_leaves_the_buffers_alone():
    n = 1000
    master = torch.ones(n, device=DEV)
    mom, var, grad = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV), torch.ones(n, device=DEV)
    inv = hb.HARLI_ERR_INVALID
    rejected(inv, hb.adamw_step, master, mom, var, grad, None, step=0)
    rejected(inv, hb.adamw_step, master, mom, var, grad, None, step=1, beta1=1.0)
    rejected(inv, hb.adamw_step, master, mom, var, grad, None, step=1, beta2=-0.1)
    rejected(inv, hb.adamw_step, master, mom, var, None, None, step=1)
    torch.cuda.synchronize()
    assert float(master.min()) == 1.0 == float(master.max()) and float(mom.abs().max()) == 0.0 and float(var.abs().max()) == 0.0
