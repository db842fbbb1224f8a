"""Limits of the finetune unit's IEEE-half arithmetic (the paper ran FP16, Sec. 8.1) and of its shapes, stated as
tests: outlier channels that half can hold leave the results at the usual bar; values it cannot hold are reported
through harli_ctx_check (or refused at attach when they are frozen weights) instead of silently clamped; a sequence
whose length is not a multiple of 8 is padded at its end by the caller, which changes nothing (causal attention)."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import harli_oracle as O
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import DEV, FinetuneCase, assert_close, shapes_of
from tests.test_finetune_gpu import check

pytestmark = pytest.mark.gpu

ALL = wl.LoraCfg(8, 16.0, wl.LORA_TARGETS)
UP_ROWS, X_COLS = (5, 100, 333), (3, 77)


def outliers(up_scale, x_scale):
    def tweak(case):
        case.W_np["wu"][list(UP_ROWS), :] *= up_scale          # a few channels of the up projection: u, m carry outliers
        case.X_np[..., list(X_COLS)] *= x_scale                # and of the residual stream the layer reads
    return tweak


def build(**kw):
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    return FinetuneCase(w, m, ALL, w.finetune, **kw)


def test_outlier_channels_inside_the_range_of_half_meet_the_usual_bar():
    """u and m = silu(a) u with channels of 1e3 .. 1e4, residual-stream outliers of the same size.  The gradients of the
    gated FFN are products with those channels: at the default gradient scale they leave half's range (reported, next
    test); with headroom they stay inside and every tensor meets the bar against the oracle."""
    case = build(tweak=outliers(5e3, 30.0), grad_headroom_log2=6)
    _, saved = O.layer_forward(case.X_np, case.W_np, case.lora_np, case.lora.scale, shapes_of(case.m))
    u_max, m_max = float(np.abs(saved["u"]).max()), float(np.abs(saved["m"]).max())
    print("oracle: max |u| %.0f, max |m| %.0f" % (u_max, m_max))
    assert 1e3 < u_max < 1e4 and 1e3 < m_max < 1e4
    check(case, "outliers inside the range")
    case.ctx.check()                                             # nothing was clamped


def test_values_beyond_the_range_of_half_are_reported_not_silently_clamped():
    # backward: the same model at the default gradient scale
    case = build(tweak=outliers(5e3, 30.0))
    case.forward_gpu()
    case.ctx.check()                                             # the forward pass fits
    _, _, dY, _, _ = case.oracle()
    case.backward_gpu(dY)
    with pytest.raises(hb.HarliError) as e:
        case.ctx.check()
    assert e.value.status == hb.HARLI_ERR_INVALID and "16-bit" in str(e.value), str(e.value)
    case.ctx.check()                                             # reported once, then clear
    # forward: activations themselves beyond 65504
    case = build(tweak=outliers(3e5, 1.0))
    Y = case.forward_gpu()
    assert np.isfinite(Y).all()                                  # clamped, never infinite
    with pytest.raises(hb.HarliError) as e:
        case.ctx.check()
    assert "16-bit" in str(e.value), str(e.value)


def test_a_frozen_weight_beyond_the_range_of_half_is_refused_at_attach():
    w = wl.workload(0)                                           # fp32 storage can hold such a weight
    assert w.model.dtype == "f32"

    def tweak(case):
        case.W_np["wd"][7, 9] = 1.0e5
    case = FinetuneCase(w, w.model, ALL, w.finetune, tweak=tweak, attach=False)
    with pytest.raises(hb.HarliError) as e:
        case.ctx.lora_attach(ALL.rank, ALL.alpha, ALL.targets, [case.A_dev], [case.B_dev])
    assert e.value.status == hb.HARLI_ERR_INVALID and "65504" in str(e.value), str(e.value)
    case.ctx.check()                                             # the refusal left no flag behind
    with pytest.raises(hb.HarliError):                           # and no half-made state: a second attach refuses again
        case.ctx.lora_attach(ALL.rank, ALL.alpha, ALL.targets, [case.A_dev], [case.B_dev])


def test_head_sizes_without_a_fused_attention_kernel_are_refused_at_attach():
    w = wl.workload(0)
    m = dataclasses.replace(w.model, hidden=128, n_q=4, n_kv=2, head_dim=32, ffn=320)   # fp32 storage decodes at any even size
    case = FinetuneCase(w, m, wl.LoraCfg(8, 16.0, ("q", "v")), wl.FinetuneCfg(1, 64), attach=False)
    with pytest.raises(hb.HarliError) as e:
        case.ctx.lora_attach(8, 16.0, ("q", "v"), [case.A_dev], [case.B_dev])
    assert e.value.status == hb.HARLI_ERR_INVALID and "head_dim" in str(e.value)


@pytest.mark.parametrize("S", [70, 121])
def test_a_ragged_sequence_padded_to_a_multiple_of_8_gives_the_results_of_the_unpadded_one(S):
    """The unit takes sequence lengths that are multiples of 8.  A caller pads each sequence at its END (any finite
    values) and gives the padded rows dY = 0: causal attention keeps the padding out of every earlier position, and
    rows with zero dY add nothing to dA, dB.  The oracle runs the unpadded sequences."""
    Sp = -(-S // 8) * 8
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    case = FinetuneCase(w, m, ALL, wl.FinetuneCfg(2, Sp))
    sh = shapes_of(m)
    X = case.X_np[:, :S]
    Y_ref, saved = O.layer_forward(X, case.W_np, case.lora_np, case.lora.scale, sh)
    _, dY = O.mse_loss(Y_ref, case.T_np[:, :S])
    dX_ref, g_ref = O.layer_backward(dY, saved, case.W_np, case.lora_np, case.lora.scale, sh)
    with pytest.raises(hb.HarliError):                           # the limit itself
        case.ctx.lora_fwd(0, case.X_dev, torch.empty(2 * S, m.hidden, device=DEV), 2, S)
    Y = case.forward_gpu()
    assert_close(Y[:, :S], Y_ref, "Y")
    dY_pad = np.zeros_like(case.X_np)
    dY_pad[:, :S] = dY
    dX, g = case.backward_gpu(dY_pad)
    assert_close(dX[:, :S], dX_ref, "dX")
    for p in g:
        assert_close(g[p][0], g_ref[p][0], "dA[%s]" % p)
        assert_close(g[p][1], g_ref[p][1], "dB[%s]" % p)
