"""GPU parity of harli_lora_fwd / harli_lora_bwd against the CPU oracle (through the C ABI).

Bar for every tensor (Y, dX, dA, dB): max-abs error <= 2e-2 * max|ref| and relative Frobenius
error <= 5e-3 (bf16 storage, fp32 accumulation).  The backward pass is fed the ORACLE's dY so
that forward error is not charged to it.
"""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import FinetuneCase, assert_close

pytestmark = pytest.mark.gpu


def build(idx=0, lora=None, ft=None, zero_b=False, **model_kw):
    w = wl.workload(idx)
    m = dataclasses.replace(w.model, dtype="bf16", **model_kw)
    return FinetuneCase(w, m, lora or w.lora, ft or w.finetune, zero_b=zero_b)


def check(case, what=""):
    from tests.gpu_util import max_abs_ratio, rel_fro
    Y = case.forward_gpu()
    refY, loss, dY, refdX, refg = case.oracle()
    r = {"Y": (max_abs_ratio(Y, refY), rel_fro(Y, refY))}
    live = case.pool.stats()
    assert live.reserved_bytes_live >= case.ctx.saved_bytes(case.ft.micro_batch, case.ft.seq_len)   # activations sit in the unified pool
    dX, g = case.backward_gpu(dY)
    r["dX"] = (max_abs_ratio(dX, refdX), rel_fro(dX, refdX))
    assert set(g) == set(refg) == set(case.lora.targets)
    for p in g:
        r["dA_" + p] = (max_abs_ratio(g[p][0], refg[p][0]), rel_fro(g[p][0], refg[p][0]))
        r["dB_" + p] = (max_abs_ratio(g[p][1], refg[p][1]), rel_fro(g[p][1], refg[p][1]))
    print(what, {k: "%.1e/%.1e" % v for k, v in r.items()})
    bad = {k: v for k, v in r.items() if not (v[0] <= 2e-2 and v[1] <= 5e-3)}      # NaN fails too
    assert not bad, "outside max-abs <= 2e-2*max|ref|, rel-Fro <= 5e-3: %s" % bad
    st = case.pool.stats()                                                     # polls the release events
    assert st.tensor_blocks_live == 0 and st.small_bytes_live == 0 and st.pending_frees == 0
    assert st.free_chunks == st.n_chunks
    return r


def test_config0_shapes_bf16():
    """hidden 256, 4 x 64 heads, ffn 688, r 8 on q and v, 2 x 128 tokens."""
    check(build(0))


def test_config0_as_written_fp32_storage():
    """Config 0 with its own storage type: fp32 weights and adapters at the ABI, rounded once to the unit's 16-bit
    compute element (the oracle uses the fp32 values), same bar."""
    w = wl.workload(0)
    assert w.model.dtype == "f32"
    check(FinetuneCase(w, w.model, w.lora, w.finetune), "config 0 fp32 storage")


def test_all_seven_targets_and_ragged_sequence():
    w = wl.workload(0)
    check(build(0, lora=wl.LoraCfg(16, 32.0, wl.LORA_TARGETS), ft=wl.FinetuneCfg(3, 72)))


@pytest.mark.parametrize("n_q,n_kv,d", [(8, 2, 64), (4, 4, 128), (8, 1, 128)])
def test_gqa_and_head_sizes(n_q, n_kv, d):
    check(build(0, lora=wl.LoraCfg(8, 16.0, ("q", "k", "v", "o")), ft=wl.FinetuneCfg(2, 96),
                hidden=n_q * d // 2, n_q=n_q, n_kv=n_kv, head_dim=d, ffn=320))


def test_long_sequence_crosses_several_tiles():
    check(build(0, ft=wl.FinetuneCfg(1, 600), lora=wl.LoraCfg(32, 64.0, ("q", "o", "down"))))


def test_zero_b_gives_base_output_and_zero_dA():
    """LoRA init property on the GPU path: with B = 0 the forward equals the base model and dA = 0 exactly."""
    case = build(0, zero_b=True)
    Y = case.forward_gpu()
    base = build(0, lora=dataclasses.replace(case.lora), zero_b=True)
    refY, _, dY, _, refg = case.oracle()
    assert_close(Y, refY, "Y")
    dX, g = case.backward_gpu(dY)
    for p in g:
        assert np.all(g[p][0] == 0.0)
        assert_close(g[p][1], refg[p][1], "dB[%s]" % p)


def test_gradients_accumulate():
    case = build(0)
    case.forward_gpu()
    _, _, dY, _, refg = case.oracle()
    case.backward_gpu(dY)
    case.forward_gpu()
    _, g2 = case.backward_gpu(dY, accumulate_into=True)
    for p in g2:
        assert_close(g2[p][0], 2 * refg[p][0], "2 dA[%s]" % p)
        assert_close(g2[p][1], 2 * refg[p][1], "2 dB[%s]" % p)


def test_forward_only_release_and_oom():
    case = build(0)
    case.forward_gpu()
    case.ctx.saved_release(case.saved)
    torch.cuda.synchronize()
    st = case.pool.stats()
    assert st.tensor_blocks_live == 0 and st.small_bytes_live == 0
    # a pool too small for the activations: HARLI_ERR_OOM and nothing left allocated
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    tight = FinetuneCase(w, m, w.lora, w.finetune, n_chunks=2, block_bytes=64 << 10, small_pool_bytes=1 << 20)
    with pytest.raises(hb.HarliError) as e:
        tight.forward_gpu()
    assert e.value.status == hb.HARLI_ERR_OOM
    st = tight.pool.stats()
    assert st.tensor_blocks_live == 0 and st.small_bytes_live == 0


def test_config1_full_size_layer():
    """The 7B-class layer: 4 x 512 tokens, r 16 on q,k,v,o."""
    w = wl.workload(1)
    case = FinetuneCase(w, w.model, w.lora, w.finetune)
    r = check(case)
    print({k: "%.1e/%.1e" % v for k, v in r.items()})


def test_config3_width_layer_rank64_all_targets():
    """13B-class layer (hidden 5120, 40 x 128 heads, ffn 13824), r 64 on all seven projections, 2 x 1024 tokens
    (half of the workload's micro-batch of 4: the oracle's time is linear in it)."""
    w = wl.workload(3)
    m = dataclasses.replace(w.model, n_layers=1)
    case = FinetuneCase(w, m, w.lora, wl.FinetuneCfg(2, 1024))
    check(case, "config 3 layer")


def test_config4_width_layer_gqa_rank32():
    """8B-class GQA layer (32 query / 8 KV heads, ffn 14336), r 32 on q,k,v,o, 4 x 512 tokens."""
    w = wl.workload(4)
    m = dataclasses.replace(w.model, n_layers=1)
    case = FinetuneCase(w, m, w.lora, wl.FinetuneCfg(4, 512))
    check(case, "config 4 layer")


def test_config5_width_layer_biases_and_groups_of_seven():
    """Qwen2.5-7B-class layer (hidden 3584, 28 query / 4 KV heads, ffn 18944, biases on q, k, v), r 16 on q,k,v,o,
    2 x 512 tokens."""
    w = wl.workload(5)
    m = dataclasses.replace(w.model, n_layers=1)
    case = FinetuneCase(w, m, w.lora, wl.FinetuneCfg(2, 512))
    assert "bq" in case.W_np
    check(case, "config 5 layer")


def test_biases_small_shape_fp32_storage_and_bf16():
    for dtype in ("bf16", "f32"):
        w = wl.workload(0)
        m = dataclasses.replace(w.model, dtype=dtype, qkv_bias=True)
        case = FinetuneCase(w, m, wl.LoraCfg(8, 16.0, ("q", "k", "v", "o")), wl.FinetuneCfg(2, 128))
        check(case, "tiny layer with biases, %s storage" % dtype)
