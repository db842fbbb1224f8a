"""Measurement hooks of the debug ABI: the read-bandwidth probe, the weight GEMM's in-kernel clock probe, the timing hook of
the decode GEMMs above 32 sequences."""
import pytest
import torch

from paper_2511_11729_amd import binding as hb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_read_bandwidth_probe_reports_sane_rates():
    """The ceilings the benchmark quotes: HBM streaming and L2-resident re-reads, both between 0.5 and 40 TB/s."""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    hbm = hb.dbg_read_bandwidth(buf, 0)
    l2 = hb.dbg_read_bandwidth(buf, 1)
    print("probe: HBM stream %.0f GB/s, L2 re-read %.0f GB/s" % (hbm, l2))
    assert 500 < hbm < 40000 and 500 < l2 < 40000 and l2 > hbm
    small = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(hb.HarliError):
        hb.dbg_read_bandwidth(small, 0)


def test_clock_probe_reports_the_clock_and_leaves_the_product_intact():
    """The in-kernel clock probe of the weight GEMM: a plausible shader clock (0.5 .. 2.6 GHz), a plausible rate, and
    the same product as the fp64 reference."""
    M, N, K = 512, 384, 256
    g = torch.Generator().manual_seed(5)
    A = ((torch.rand(M, K, generator=g) - 0.5)).half().to(DEV)
    B = ((torch.rand(N, K, generator=g) - 0.5)).half().to(DEV)
    Cb = torch.empty(M, N, dtype=torch.float16, device=DEV)
    tf, mhz = hb.dbg_gemm2(M, [{"A": A, "B": B}], [{"N": N, "cb": Cb}], half=True, reps=3)
    assert 500.0 < mhz < 2600.0 and tf > 0.0
    ref = A.double().cpu() @ B.double().cpu().T
    assert float((Cb.double().cpu() - ref).abs().max()) <= 2e-3 * float(ref.abs().max())


def test_decode_gemm_timing_hook_runs_the_cut_it_is_asked_for():
    """harli_dbg_decode_gemm_time: the plan's own cut, a forced number of K ranges, the SwiGLU pair; times are positive and
    the hook gives the choice back afterwards."""
    own = hb.dbg_decode_gemm_time(150, 1024, 1, 2048, 0, 3)
    assert own["gemm_us"] > 0 and own["epilogue_us"] > 0 and own["FM"] == 3
    assert own["ksplit"] == hb.dbg_decode_gemm_plan(150, 1024, 1, 2048, torch.cuda.get_device_properties(0).multi_processor_count, 192 << 20)["ksplit"]
    forced = hb.dbg_decode_gemm_time(150, 1024, 1, 2048, 3, 3)
    assert forced["ksplit"] == 3
    pair = hb.dbg_decode_gemm_time(40, 688, 2, 256, 0, 3)            # a ragged last weight tile, one K range
    assert pair["ksplit"] == 1 and pair["FM"] == 1 and pair["gemm_us"] > 0
    again = hb.dbg_decode_gemm_time(150, 1024, 1, 2048, 0, 3)
    assert again["ksplit"] == own["ksplit"]
    with pytest.raises(hb.HarliError):
        hb.dbg_decode_gemm_time(150, 1023, 1, 2048, 0, 3)             # rows must be a multiple of 8
