"""Compute-unit partitions and the predictor on the device: a decode step on a CU-range stream gives the same
result as on an ordinary stream, profiling yields a usable Eq. 1 / Eq. 2 fit, and the chosen partition keeps
the decode time per output token inside the SLO while finetune units run beside it."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import harli_oracle as O
from paper_2511_11729_amd import binding as hb
from paper_2511_11729_amd import colocate
from paper_2511_11729_amd.harness import LayerHarness
from tests.gpu_util import assert_close, shapes_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hz():
    return LayerHarness(wl.workload(1), in_flight=8, decode_capacity=(64, 2048))


def test_cu_range_stream_validates_its_range():
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for first, count in [(-1, 4), (0, 0), (n_cu, 1), (8, n_cu)]:
        with pytest.raises(hb.HarliError) as e:
            hb.cu_stream_create(first, count)
        assert e.value.status == hb.HARLI_ERR_INVALID
    s = hb.cu_stream_create(n_cu - 8, 8)
    hb.cu_stream_destroy(s)


def test_decode_on_a_quarter_of_the_chip_matches_the_full_chip(hz):
    cs = colocate.CuStreams()
    full = torch.cuda.Stream()
    part = cs.low(3)                                   # 30 % of the compute units
    hz.decode_launch(full)
    full.synchronize()
    want = hz.y_dev[: hz.B].clone()
    hz.y_dev.zero_()
    hz.decode_launch(part)
    part.synchronize()
    hz.ctx.check(part)
    got = hz.y_dev[: hz.B]
    # same kernels, same inputs, no arithmetic that depends on how many workgroups run at a time: the same bits,
    # and the oracle's result at the bf16 bar in this launch configuration too
    assert torch.equal(got, want)
    x_np, _, kv_np = wl.make_decode_inputs(hz.w)
    yo, _ = O.decode_layer_contiguous(x_np, hz.W_np, shapes_of(hz.m), kv_np[0])
    assert_close(got.cpu().numpy(), yo, "decode on 3/10 of the compute units")
    t_full = colocate.time_decode(hz, full, None, None, None, 10)
    t_part = colocate.time_decode(hz, part, None, None, None, 10)
    assert t_part > 1.3 * t_full                       # the restriction is real
    hz.drain()
    cs.close()


def test_finetune_unit_on_a_partition_is_bit_identical_and_slower(hz):
    cs = colocate.CuStreams()
    full = torch.cuda.Stream()
    part = cs.high(4)                                  # the last 40 % of the compute units

    def unit_on(st):
        for p in hz.dA:
            hz.dA[p].zero_()
            hz.dB[p].zero_()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        hz.finetune_unit(st)
        e1.record(st)
        st.synchronize()
        hz.drain()
        out = (hz.Y_dev.clone(), hz.dX_dev.clone(), {p: hz.dA[p].clone() for p in hz.dA}, {p: hz.dB[p].clone() for p in hz.dB})
        torch.cuda.synchronize()
        return out, e0.elapsed_time(e1)

    unit_on(full)                                      # first use sizes the workspace
    (Y1, dX1, dA1, dB1), t_full = unit_on(full)
    (Y2, dX2, dA2, dB2), t_part = unit_on(part)
    hz.ctx.check(part)
    # no kernel of the unit depends on how many workgroups run at a time
    assert torch.equal(Y1, Y2) and torch.equal(dX1, dX2)
    assert all(torch.equal(dA1[p], dA2[p]) and torch.equal(dB1[p], dB2[p]) for p in dA1)
    assert t_part > 1.5 * t_full                       # 40 % of the chip: the restriction is real
    cs.close()


def test_profile_fit_and_scheduled_colocation(hz):
    pred, rep = colocate.profile(hz, steps=6)
    solo = rep["solo_ms_by_level_workload_batch"]
    assert solo[0] > 2.0 * solo[-1]                    # a tenth of the chip is much slower than all of it
    assert all(solo[i + 1] <= 1.15 * solo[i] for i in range(9))
    assert rep["eq1_mean_abs_err_heldout"] < 0.20      # Eq. 1 describes decode latency on every partition
    b0, c0, k0 = rep["eq1_coef_full_chip_b0_c0_k0_ms"]
    assert c0 > 0 and k0 > 0                           # a weight-streaming floor and a per-token cost
    slo = 40.0 / 32.0
    il, fl, plat = pred.pick(hz.B, int(hz.kv_len.mean()), slo)
    assert 1 <= il <= 10 and 0 <= fl <= 10 - il and (fl == 0 or plat <= slo)
    cs = colocate.CuStreams()
    low, high = cs.pairs()                             # streams on different dispatch pipes
    sD, sF = low[il], high[max(fl, 1)]
    res = colocate.run_colocated(hz, sD, sF, lambda: hz.decode_launch(sD), 4, 1, None)
    hz.ctx.check(sD)
    hz.drain()                                         # no event of the harness outlives the streams
    cs.close()
    assert res["tokens_per_s"] > 0
    assert float(np.percentile(res["tpot"], 99)) <= slo
    st = hz.pool.stats()
    assert st.pending_frees == 0 or st.pending_frees <= 16


def test_runtime_scheduler_replays_a_load_trace(hz):
    """Light -> heavy -> medium decode load (the shape of the paper's memory/SM-ratio traces, Sec. 8.5-8.6) with two
    starvation episodes: the decode step stays inside the target in nearly every phase, the finetune task makes
    progress in every segment, starved phases give inference the whole chip, and a heavier load never gets a
    smaller inference share."""
    pred, _ = colocate.profile(hz, steps=6)
    slo = 40.0 / 32.0
    segs = [(40, 8), (40, 42), (40, 24)]
    starve = set(range(20, 24)) | set(range(100, 103))
    out = colocate.run_trace(hz, pred, slo, segs, seqlen=1024, refresh_phases=16, starve=starve, log=print)
    ph, sg = out["phases"], out["segments"]
    assert len(ph) == 120
    for r in ph:
        if r["phase"] in starve:
            assert (r["infer_level"], r["ft_level"], r["action"]) == (10, 0, hb.SCHED_STARVED)
        else:
            assert r["infer_level"] + r["ft_level"] <= 10 and r["infer_level"] >= 1
            assert r["ft_level"] == 0 or r["predicted_ms"] <= slo
    for s in sg:
        assert s["within_slo"] >= 0.85, s              # the first phases of a segment may miss until the measured correction settles
        assert s["finetune_units"] >= 1, s
    light = min(i for i, f in sg[0]["plans"] if f > 0)
    heavy = min(i for i, f in sg[1]["plans"] if f > 0)
    assert heavy >= light
    # the phase after a starvation episode re-plans
    assert ph[24]["action"] == hb.SCHED_REPLAN and ph[103]["action"] == hb.SCHED_REPLAN
    torch.cuda.synchronize()                          # units the feeder issued last may still be running
    assert hz.pool.stats().pending_frees == 0          # every saved activation went back once its unit was done
