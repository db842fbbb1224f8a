"""The finetune unit's weight GEMM (256-wide tiles, weight side in blocked order, direct-to-LDS loads) on its own, through
the C ABI's test hook, against an fp64 product of the same 16-bit inputs: ragged M / N / K, K segments shorter than a
K step (the LoRA path), several output blocks in one launch (q, k, v), the interleaved gate/up pair with its SwiGLU
epilogue, the SwiGLU backward epilogue, fp32 output with a residual, both tile heights and both element types."""
import numpy as np
import pytest
import torch

from paper_2511_11729_amd import binding as hb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dt(half):
    return torch.float16 if half else torch.bfloat16


def rnd(shape, half, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dt(half)).to(DEV)


def f64(t):
    return t.detach().cpu().double().numpy()


def close(got, ref, what, rel=2e-3):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref).max()
    assert err <= rel * np.abs(ref).max() + 1e-6, "%s: max err %.3e vs max |ref| %.3e" % (what, err, np.abs(ref).max())


@pytest.mark.parametrize("half", [True, False])
@pytest.mark.parametrize("tile_rows", [128, 256])
@pytest.mark.parametrize("M,N,K,K2", [(300, 520, 200, 16), (64, 256, 32, 0), (513, 1000, 4096 + 8, 64), (257, 8, 8, 8)])
def test_plain_product_with_a_short_second_segment(half, tile_rows, M, N, K, K2):
    A, B = rnd((M, K), half, 1), rnd((N, K), half, 2, 0.1)
    segs = [dict(A=A, B=B)]
    ref = f64(A) @ f64(B).T
    if K2:
        A2, B2 = rnd((M, K2), half, 3), rnd((N, K2), half, 4, 0.1)
        segs.append(dict(A=A2, B=B2))
        ref = ref + f64(A2) @ f64(B2).T
    cb = torch.full((M, N), float("nan"), dtype=dt(half), device=DEV)
    hb.dbg_gemm2(M, segs, [dict(N=N, cb=cb)], half=half, alpha=0.5, tile_rows=tile_rows)
    close(f64(cb), 0.5 * ref, "16-bit output", 2e-3 if half else 1e-2)
    # fp32 output with a residual (and a 16-bit copy), same operands
    res = torch.randn(M, N, device=DEV)
    ldc = (N + 3) // 4 * 4
    cf = torch.full((M, ldc), float("nan"), device=DEV)
    resp = torch.zeros(M, ldc, device=DEV)
    resp[:, :N] = res
    hb.dbg_gemm2(M, segs, [dict(N=N, cf=cf, res=resp, ld=ldc)], half=half, tile_rows=tile_rows)
    close(f64(cf[:, :N]), ref + f64(res), "fp32 output + residual", 1e-5)
    assert torch.isnan(cf[:, N:]).all()                     # nothing is written past the last valid column


@pytest.mark.parametrize("tile_rows", [128, 256])
def test_three_output_blocks_with_an_adapter_on_two_of_them(tile_rows):
    """q, k, v in one launch: blocks of 512, 256 and 200 columns (the last one ragged), a rank-16 adapter segment on the
    first and the third only, a frozen-bias segment (K = 8) on all."""
    half, M, H, r = True, 333, 384, 16
    Ns = [512, 256, 200]
    h = rnd((M, H), half, 10)
    W = [rnd((n, H), half, 11 + i, 0.05) for i, n in enumerate(Ns)]
    us = {0: rnd((M, r), half, 20), 2: rnd((M, r), half, 21)}
    Bt = {0: rnd((Ns[0], r), half, 22, 0.1), 2: rnd((Ns[2], r), half, 23, 0.1)}
    ones = torch.ones(M, 8, dtype=dt(half), device=DEV)
    bias = [torch.zeros(n, 8, dtype=dt(half), device=DEV) for n in Ns]
    for i, n in enumerate(Ns):
        bias[i][:, 0] = rnd((n,), half, 30 + i)
    t0 = [0, 2, 3]
    t1 = [2, 3, 4]
    segs, outs, cbs = [], [], []
    for i, n in enumerate(Ns):
        segs.append(dict(A=h, B=W[i], tile0=t0[i], tile1=t1[i]))
        segs.append(dict(A=ones, B=bias[i], tile0=t0[i], tile1=t1[i]))
        if i in us:
            segs.append(dict(A=us[i], B=Bt[i], tile0=t0[i], tile1=t1[i]))
        cb = torch.full((M, n), float("nan"), dtype=dt(half), device=DEV)
        cbs.append(cb)
        outs.append(dict(N=n, cb=cb, tile0=t0[i]))
    hb.dbg_gemm2(M, segs, outs, half=half, tile_rows=tile_rows)
    for i, n in enumerate(Ns):
        ref = f64(h) @ f64(W[i]).T + f64(bias[i][:, 0])[None, :]
        if i in us:
            ref = ref + f64(us[i]) @ f64(Bt[i]).T
        close(f64(cbs[i]), ref, "block %d" % i)


@pytest.mark.parametrize("half", [True, False])
@pytest.mark.parametrize("M,F,H", [(300, 384, 256), (129, 200, 72), (512, 11008 // 8, 512)])
def test_gate_up_pair_with_swiglu_epilogue_and_its_backward(half, M, F, H):
    r = 8
    h2 = rnd((M, H), half, 40)
    Wg, Wu = rnd((F, H), half, 41, 0.08), rnd((F, H), half, 42, 0.08)
    usg, usu = rnd((M, r), half, 43), rnd((M, r), half, 44)
    Bg, Bu = rnd((F, r), half, 45, 0.1), rnd((F, r), half, 46, 0.1)
    a = torch.full((M, F), float("nan"), dtype=dt(half), device=DEV)
    u, m = torch.full_like(a, float("nan")), torch.full_like(a, float("nan"))
    segs = [dict(A=h2, B=Wg, B2=Wu, pair=1), dict(A=usg, B=Bg, B2=None, pair=1), dict(A=usu, B=None, B2=Bu, pair=1)]
    hb.dbg_gemm2(M, segs, [dict(N=F, cb=a)], half=half, epi=3, o0=m, o1=u, lde=F)
    a_ref = f64(h2) @ f64(Wg).T + f64(usg) @ f64(Bg).T
    u_ref = f64(h2) @ f64(Wu).T + f64(usu) @ f64(Bu).T
    tol = 2e-3 if half else 1e-2
    close(f64(a), a_ref, "gate", tol)
    close(f64(u), u_ref, "up", tol)
    ar, ur = f64(a), f64(u)                                   # m is formed from the rounded a and u
    close(f64(m), ar / (1 + np.exp(-ar)) * ur, "silu(a) * u", tol)
    # backward epilogue: dm = dy Wd^T-like product, da and du from the stored a, u
    dy = rnd((M, H), half, 47)
    WdT = rnd((F, H), half, 48, 0.08)
    da, du = torch.full_like(a, float("nan")), torch.full_like(a, float("nan"))
    hb.dbg_gemm2(M, [dict(A=dy, B=WdT)], [dict(N=F)], half=half, epi=2, e0=a, e1=u, o0=da, o1=du, lde=F)
    dm = f64(dy) @ f64(WdT).T
    sg = 1 / (1 + np.exp(-ar))
    close(f64(da), dm * ur * sg * (1 + ar * (1 - sg)), "da", tol)
    close(f64(du), dm * ar * sg, "du", tol)


def test_an_output_beyond_the_range_of_half_sets_the_flag():
    M, N, K = 128, 256, 64
    A = torch.full((M, K), 200.0, dtype=torch.float16, device=DEV)
    B = torch.full((N, K), 200.0, dtype=torch.float16, device=DEV)      # every output is 2.56e6 > 65504
    cb = torch.zeros(M, N, dtype=torch.float16, device=DEV)
    flag = torch.zeros(4, dtype=torch.int32, device=DEV)
    hb.dbg_gemm2(M, [dict(A=A, B=B)], [dict(N=N, cb=cb)], half=True, overflow_flag=flag)
    assert int(flag[0]) & 8 and float(cb.max()) == 65504.0
    flag.zero_()
    hb.dbg_gemm2(M, [dict(A=A, B=B)], [dict(N=N, cb=cb)], half=True, alpha=1e-3, overflow_flag=flag)
    assert int(flag[0]) == 0


def test_full_size_shapes_on_sampled_outputs():
    """The shapes of the 7B-class layer at 2048 and 4096 tokens in the launch configuration the library picks, checked
    on sampled rows against fp64 dot products (the timing is printed for the record)."""
    for (M, N, K) in [(2048, 4096, 4096), (2048, 12288, 4096), (2048, 4096, 11008), (4096, 4096, 4096)]:
        A, B = rnd((M, K), True, 60, 0.5), rnd((N, K), True, 61, 0.05)
        cb = torch.empty(M, N, dtype=torch.float16, device=DEV)
        t, mhz = hb.dbg_gemm2(M, [dict(A=A, B=B)], [dict(N=N, cb=cb)], half=True, reps=10)
        rows = [0, 1, 255, 256, M // 2 + 7, M - 1]
        ref = f64(A[rows]) @ f64(B).T
        close(f64(cb[rows]), ref, "%dx%dx%d" % (M, N, K))
        print("gemm2 %d x %d x %d: %.0f TFLOP/s at %.0f MHz" % (M, N, K, t, mhz))


# ---- tile height chosen for the compute units of the stream ------------------------------------------------------------
def test_full_size_shapes_on_a_nine_tenths_partition():
    """2048 x 4096 x 4096 on a stream masked to 230 compute units: 256 tiles of 128 rows would run as one full round
    and 26 stragglers, so the library takes 128 tiles of 256 rows there (one round); sampled rows against fp64,
    timings of both tile heights on the partition for the record."""
    M, N, K = 2048, 4096, 4096
    assert hb.dbg_gemm2_plan(M, N // 256, 128, 230)["rounds"] == 2 and hb.dbg_gemm2_plan(M, N // 256, 256, 230)["rounds"] == 1
    A, B = rnd((M, K), True, 60, 0.5), rnd((N, K), True, 61, 0.05)
    rows = [0, 1, 255, 256, M // 2 + 7, M - 1]
    ref = f64(A[rows]) @ f64(B).T
    st = hb.cu_stream_create(0, 230)
    try:
        for name, kw in (("library's choice", {}), ("128-row tiles", dict(tile_rows=128)), ("256-row tiles", dict(tile_rows=256))):
            cb = torch.zeros(M, N, dtype=torch.float16, device=DEV)
            torch.cuda.synchronize()
            t, _ = hb.dbg_gemm2(M, [dict(A=A, B=B)], [dict(N=N, cb=cb)], half=True, reps=10, stream=st, **kw)
            torch.cuda.synchronize()
            close(f64(cb[rows]), ref, name)
            print("gemm2 2048 x 4096 x 4096 on 230 compute units, %s: %.0f TFLOP/s" % (name, t))
    finally:
        hb.cu_stream_destroy(st)
