"""Parity in the launch configuration the benchmark times: the benchmark's workload (config 1, full layer width), a decode
loop on one stream while finetune units run on another, both through the C ABI and from two host threads.

Sharing the chip must not change a result.  Neither task has order-dependent arithmetic (the decode step adds its
row norms across workgroups as integers), so the outputs of both beside the other are bit-identical to their outputs
alone, and both meet the oracle at the usual bar (max-abs error <= 2e-2 * max|ref|, relative Frobenius error <= 5e-3)
in this launch configuration.
"""
import threading

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import harli_oracle as O
from paper_2511_11729_amd.harness import LayerHarness
from tests.gpu_util import assert_close, shapes_of

pytestmark = pytest.mark.gpu

UNITS, DECODE_STEPS = 4, 80


def test_results_do_not_change_when_both_tasks_share_the_chip():
    w = wl.workload(1)
    hz = LayerHarness(w)
    m, T, H = hz.m, hz.T, hz.m.hidden
    sh = shapes_of(m)
    _, T_np = wl.make_finetune_inputs(w)
    Yo, sv = O.layer_forward(hz.X_np, hz.W_np, hz.lora_np, hz.lora.scale, sh)
    _, dYo = O.mse_loss(Yo, T_np)
    dXo, grads_o = O.layer_backward(dYo, sv, hz.W_np, hz.lora_np, hz.lora.scale, sh)
    hz.dY_dev.copy_(torch.from_numpy(np.ascontiguousarray(dYo.reshape(T, H), np.float32)))
    x_np, _, kv_np = wl.make_decode_inputs(w)            # what the harness put on the device
    yo, _ = O.decode_layer_contiguous(x_np, hz.W_np, sh, kv_np[0])
    sD, sF = torch.cuda.Stream(), torch.cuda.Stream()

    def zero_grads():
        for p in hz.dA:
            hz.dA[p].zero_()
            hz.dB[p].zero_()
        torch.cuda.synchronize()

    def snapshot():
        return (hz.Y_dev.clone(), hz.dX_dev.clone(), {p: hz.dA[p].clone() for p in hz.dA}, {p: hz.dB[p].clone() for p in hz.dB})

    # ---- each task alone
    zero_grads()
    for _ in range(UNITS):
        hz.finetune_unit(sF)
    sF.synchronize()
    hz.drain()
    Y1, dX1, dA1, dB1 = snapshot()
    hz.decode_launch(sD)
    sD.synchronize()
    y1 = hz.y_dev.clone()
    torch.cuda.synchronize()

    # ---- side by side: a host thread issues decode steps while this one issues finetune units
    zero_grads()
    hz.y_dev.zero_()
    torch.cuda.synchronize()
    ev = {k: torch.cuda.Event(enable_timing=True) for k in ("d0", "d1", "f0", "f1")}
    err = []

    def decode_loop():
        try:
            ev["d0"].record(sD)
            for _ in range(DECODE_STEPS):
                hz.decode_launch(sD)
            ev["d1"].record(sD)
        except Exception as e:                      # surfaces in the main thread below
            err.append(e)

    th = threading.Thread(target=decode_loop)
    th.start()
    ev["f0"].record(sF)
    for _ in range(UNITS):
        hz.finetune_unit(sF)
    ev["f1"].record(sF)
    th.join()
    sD.synchronize()
    sF.synchronize()
    hz.drain()
    assert not err, err
    hz.ctx.check(sD)
    # the two really ran at the same time: each started before the other ended
    assert ev["d0"].elapsed_time(ev["f1"]) > 0 and ev["f0"].elapsed_time(ev["d1"]) > 0
    Y2, dX2, dA2, dB2 = snapshot()

    assert torch.equal(Y1, Y2) and torch.equal(dX1, dX2)
    for p in dA1:
        assert torch.equal(dA1[p], dA2[p]) and torch.equal(dB1[p], dB2[p]), p
    assert torch.equal(hz.y_dev, y1)
    assert_close(y1[: hz.B].cpu().numpy(), yo, "decode alone")
    assert_close(hz.y_dev[: hz.B].cpu().numpy(), yo, "decode beside finetune")

    assert_close(Y2.cpu().numpy().reshape(Yo.shape), Yo, "Y beside decode")
    assert_close(dX2.cpu().numpy().reshape(dXo.shape), dXo, "dX beside decode")
    for p, (gA, gB) in grads_o.items():
        assert_close(dA2[p].cpu().numpy(), UNITS * gA, "dA[%s] beside decode" % p)
        assert_close(dB2[p].cpu().numpy(), UNITS * gB, "dB[%s] beside decode" % p)
