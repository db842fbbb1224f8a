"""The finetune unit's bf16 MFMA GEMM in isolation, against an fp64 product of the same bf16 inputs.

Inputs are exactly representable, accumulation is fp32, so the fp32 output must agree to fp32
round-off of a K-term sum; the bf16 outputs to one bf16 rounding.
"""
import pytest
import torch

from paper_2511_11729_amd import binding as hb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


DT = torch.bfloat16


def rnd(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(DT).to(DEV)


@pytest.fixture(params=["half", "bf16"], autouse=True)
def operand_type(request):
    global DT
    DT = torch.float16 if request.param == "half" else torch.bfloat16
    yield request.param


@pytest.mark.parametrize("M,N,K1,K2", [
    (256, 128, 64, 0), (300, 200, 72, 0), (17, 9, 8, 0), (512, 512, 128, 16), (2048, 4096, 4096, 16),
    (2048, 11008, 4096, 0), (2048, 4096, 11008, 0), (1000, 136, 264, 8),
])
def test_gemm_matches_fp64(M, N, K1, K2):
    A1, B1 = rnd((M, K1), 1), rnd((N, K1), 2, 0.05)
    A2 = rnd((M, K2), 3) if K2 else None
    B2 = rnd((N, K2), 4, 0.05) if K2 else None
    res = torch.randn(M, N, device=DEV)
    Cb = torch.zeros(M, N, dtype=DT, device=DEV)
    Cf = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    Ct = torch.zeros(N, M, dtype=DT, device=DEV)
    hb.dbg_gemm(A1, B1, A2=A2, B2=B2, alpha=0.5, half=DT == torch.float16, Cb=Cb, Cf=Cf, res=res, Ct=Ct)
    torch.cuda.synchronize()
    ref = A1.double().cpu() @ B1.double().cpu().T
    if K2:
        ref = ref + A2.double().cpu() @ B2.double().cpu().T
    ref = 0.5 * ref + res.double().cpu()
    scale = float(ref.abs().max())
    err = float((Cf.double().cpu() - ref).abs().max())
    assert err <= 2e-5 * scale + 1e-6, (err, scale)
    # bf16 outputs are the fp32 result (incl. residual) rounded once
    assert torch.equal(Cb.cpu(), Cf.to(DT).cpu())
    assert torch.equal(Ct.cpu(), Cf.to(DT).cpu().T.contiguous())


@pytest.mark.parametrize("causal", [1, 2, 3, 4])
def test_causal_modes(causal):
    S, d = 600, 64
    if causal in (1, 2):                       # S x S output from [S, d] operands
        A, B = rnd((S, d), 5), rnd((S, d), 6)
        Cf = torch.full((S, S), 7.0, dtype=torch.float32, device=DEV)
        hb.dbg_gemm(A, B, causal=causal, half=DT == torch.float16, Cf=Cf)
        torch.cuda.synchronize()
        ref = (A.double() @ B.double().T).cpu()
        got = Cf.double().cpu()
        keep = torch.tril(torch.ones(S, S, dtype=torch.bool)) if causal == 1 else torch.triu(torch.ones(S, S, dtype=torch.bool))
        assert float((got - ref)[keep].abs().max()) <= 1e-4 * float(ref.abs().max())
        # skipped tiles keep their previous contents; computed ones outside the triangle hold the true product
        other = got[~keep]
        assert bool(((other == 7.0) | ((other - ref[~keep]).abs() <= 1e-4 * float(ref.abs().max()))).all())
    else:                                      # triangular A [S, S] times B [d, S]
        tri = torch.tril if causal == 3 else torch.triu
        A = tri(rnd((S, S), 8).float()).to(DT)
        B = rnd((d, S), 9)
        Cf = torch.zeros(S, d, dtype=torch.float32, device=DEV)
        hb.dbg_gemm(A, B, causal=causal, half=DT == torch.float16, Cf=Cf)
        torch.cuda.synchronize()
        ref = (A.double() @ B.double().T).cpu()
        assert float((Cf.double().cpu() - ref).abs().max()) <= 1e-4 * float(ref.abs().max())


def test_bad_arguments_are_rejected():
    A, B = rnd((16, 12), 1), rnd((16, 12), 2)          # K not a multiple of 8
    with pytest.raises(hb.HarliError):
        hb.dbg_gemm(A, B, Cf=torch.zeros(16, 16, device=DEV))
    A, B = rnd((16, 16), 1), rnd((16, 16), 2)
    with pytest.raises(hb.HarliError):
        hb.dbg_gemm(A, B)                                  # no output


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
    """The in-kernel clock probe: a plausible shader clock (0.5 .. 2.6 GHz), a plausible rate, and the same product
    as the fp64 reference."""
    M, N, K = 512, 384, 256
    g = torch.Generator().manual_seed(5)
    A = ((torch.rand(M, K, generator=g) - 0.5)).half().to(DEV)
    B = ((torch.rand(N, K, generator=g) - 0.5)).half().to(DEV)
    Cb = torch.empty(M, N, dtype=torch.float16, device=DEV)
    tf, mhz = hb.dbg_gemm_clock(A, B, Cb, half=True, reps=3)
    assert 500.0 < mhz < 2600.0 and tf > 0.0
    ref = A.double().cpu() @ B.double().cpu().T
    assert float((Cb.double().cpu() - ref).abs().max()) <= 2e-3 * float(ref.abs().max())
    with pytest.raises(hb.HarliError):
        hb.dbg_gemm_clock(A, B, Cb, half=True, reps=0)
