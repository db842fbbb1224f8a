"""Device memory of the library: what a context holds is reported, the finetune task's workspace can live in the unified
pool (Sec. 4.2: one pool for every tensor of both tasks) where the pool's statistics see it, results do not depend on
where it lives, and a finetune unit allocates no device memory once the adapters are attached."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import DEV, FinetuneCase, assert_close, f32_dev, to_dev

pytestmark = pytest.mark.gpu


def unit(fc, dY):
    Y = fc.forward_gpu()
    dX, grads = fc.backward_gpu(dY)
    return Y, dX, grads


def test_workspace_in_the_pool_is_accounted_and_changes_no_result():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    fc = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=64)        # roomy: 64 chunks of 4 MiB
    _, _, dY, dX_ref, grads_ref = fc.oracle()
    b0 = fc.ctx.device_bytes()
    assert b0.in_pool == 0 and b0.finetune_workspace > 0 and b0.finetune_weights > 0 and b0.decode_weights > 0
    assert b0.outside_pool == (b0.decode_weights + b0.decode_workspace + b0.finetune_weights + b0.finetune_workspace
                               + b0.head_weights + b0.head_workspace)
    live0 = fc.pool.stats().tensor_blocks_live
    Y1, dX1, g1 = unit(fc, dY)
    # the same adapters again, now with the workspace taken from the pool
    fc.ctx.lora_attach(fc.lora.rank, fc.lora.alpha, fc.lora.targets, [fc.A_dev], [fc.B_dev], workspace_in_pool=True)
    b1 = fc.ctx.device_bytes()
    assert b1.in_pool == b1.finetune_workspace == b0.finetune_workspace
    assert b1.outside_pool == b0.outside_pool - b0.finetune_workspace
    st = fc.pool.stats()
    blocks = -(-b1.finetune_workspace // (2 << 20))
    assert st.tensor_blocks_live - live0 == blocks                  # the pool sees every block of it
    free_before = torch.cuda.mem_get_info()[0]
    Y2, dX2, g2 = unit(fc, dY)
    Y3, dX3, g3 = unit(fc, dY)
    assert torch.cuda.mem_get_info()[0] >= free_before              # no unit call allocated device memory
    assert np.array_equal(Y1, Y2) and np.array_equal(dX1, dX2) and np.array_equal(Y2, Y3) and np.array_equal(dX2, dX3)
    for p in g1:
        assert np.array_equal(g1[p][0], g2[p][0]) and np.array_equal(g1[p][1], g2[p][1])
    assert_close(dX2, dX_ref, "dX with the workspace in the pool")
    for p, (gA, gB) in grads_ref.items():
        assert_close(g2[p][0], gA, "dA[%s]" % p)
        assert_close(g2[p][1], gB, "dB[%s]" % p)
    # back to a library allocation: the pool gets its blocks back
    fc.ctx.lora_attach(fc.lora.rank, fc.lora.alpha, fc.lora.targets, [fc.A_dev], [fc.B_dev], workspace_in_pool=False)
    torch.cuda.synchronize()
    assert fc.pool.stats().tensor_blocks_live == live0 and fc.ctx.device_bytes().in_pool == 0


def test_a_pool_without_room_for_the_workspace_refuses_the_attach_and_the_next_attach_works():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    fc = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=48)
    need = fc.ctx.device_bytes().finetune_workspace
    assert need < 40 * (4 << 20)                                     # the empty pool could hold it
    # fill the chunks open to tensors (one of the eight is the inference reserve) until less than the workspace is left
    taken = []
    while True:
        try:
            taken.append(fc.pool.alloc(hb.CLS_TENSOR, 2 << 20))
        except hb.HarliError:
            break
    for _ in range(min(len(taken), max(-(-need // (2 << 20)) - 1, 0))):   # one block short of what the workspace needs
        fc.pool.free(taken.pop())
    with pytest.raises(hb.HarliError) as e:
        fc.ctx.lora_attach(fc.lora.rank, fc.lora.alpha, fc.lora.targets, [fc.A_dev], [fc.B_dev], workspace_in_pool=True)
    assert e.value.status == hb.HARLI_ERR_OOM
    Y = torch.empty(fc.ft.tokens, m.hidden, dtype=torch.float32, device=DEV)
    with pytest.raises(hb.HarliError) as e:                          # no adapters are attached now
        fc.ctx.lora_fwd(0, fc.X_dev, Y, fc.ft.micro_batch, fc.ft.seq_len)
    assert e.value.status == hb.HARLI_ERR_STATE
    for a in taken:
        fc.pool.free(a)
    fc.ctx.lora_attach(fc.lora.rank, fc.lora.alpha, fc.lora.targets, [fc.A_dev], [fc.B_dev], workspace_in_pool=True)
    _, _, dY, dX_ref, _ = fc.oracle()
    _, dX, _ = unit(fc, dY)
    assert_close(dX, dX_ref, "dX after the refused attach")


def test_pool_and_context_may_be_destroyed_in_either_order():
    """A context whose workspace lives in the pool returns it when it is destroyed; the pool object outlives its
    creator's destroy call until then (the garbage collector finalises the two Python objects in no fixed order)."""
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    fc = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=64)
    fc.ctx.lora_attach(fc.lora.rank, fc.lora.alpha, fc.lora.targets, [fc.A_dev], [fc.B_dev], workspace_in_pool=True)
    assert fc.ctx.device_bytes().in_pool > 0
    # the C-ABI order a careless caller may take: the pool first, the context after it
    h_pool, h_ctx = fc.pool.handle, fc.ctx.handle
    fc.pool.handle = type(h_pool)()
    fc.ctx.handle = type(h_ctx)()
    hb.lib().harli_pool_destroy(h_pool)
    hb.lib().harli_ctx_destroy(h_ctx)
    # the same through the binding's objects
    fc2 = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=64)
    fc2.ctx.lora_attach(fc2.lora.rank, fc2.lora.alpha, fc2.lora.targets, [fc2.A_dev], [fc2.B_dev], workspace_in_pool=True)
    fc2.pool.close()
    fc2.ctx.close()


def test_all_library_memory_in_the_pool_is_accounted_and_changes_no_result():
    """memory_in_pool: the decode instance's weight copies and step buffers, the finetune instance's weight copies and
    both workspaces are allocations of the unified pool (Sec. 4.2); the pool's statistics cover every byte the context
    reports, nothing is left outside, results are the bits of a context that allocates for itself, and destroying the
    context gives everything back."""
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    ref = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=64)
    _, _, dY, _, _ = ref.oracle()
    Y0, dX0, g0 = unit(ref, dY)
    fc = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=96, memory_in_pool=True)
    b = fc.ctx.device_bytes()
    assert b.outside_pool == 0 and b.in_pool == (b.decode_weights + b.decode_workspace + b.finetune_weights
                                                 + b.finetune_workspace + b.head_weights + b.head_workspace) > 0
    st = fc.pool.stats()
    assert st.reserved_bytes_live >= b.in_pool and st.requested_bytes_live >= b.in_pool
    assert ref.ctx.device_bytes().outside_pool == b.in_pool       # the same buffers, only placed elsewhere
    Y1, dX1, g1 = unit(fc, dY)
    assert np.array_equal(Y0, Y1) and np.array_equal(dX0, dX1)
    for p in g0:
        assert np.array_equal(g0[p][0], g1[p][0]) and np.array_equal(g0[p][1], g1[p][1])
    fc.ctx.check()
    fc.ctx.close()
    torch.cuda.synchronize()
    st = fc.pool.stats()
    assert st.tensor_blocks_live == 0 and st.small_bytes_live == 0 and st.free_chunks == st.n_chunks


def test_decode_from_pool_memory_gives_the_same_step_and_a_full_pool_refuses_the_context():
    from tests.gpu_util import DecodeCase
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    lengths = [70, 121, 64, 99]
    a = DecodeCase(w, m, lengths)
    b = DecodeCase(w, m, lengths, extra_chunks=24, memory_in_pool=True)
    ya, yb = a.run_gpu(), b.run_gpu()
    assert np.array_equal(np.asarray(ya), np.asarray(yb))
    assert b.ctx.device_bytes().outside_pool == 0 and b.pool.stats().tensor_blocks_live > 0
    with pytest.raises(hb.HarliError) as e:                      # one spare chunk cannot hold the weight copies
        DecodeCase(w, m, lengths, extra_chunks=1, memory_in_pool=True)
    assert e.value.status == hb.HARLI_ERR_OOM
