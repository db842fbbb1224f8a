"""Host logic of the large-batch decode GEMMs (harli_dbg_decode_gemm_plan): how a GEMM with M = batch is cut into batch
tiles, 256-row weight tiles and ranges of K, and what workspace the partial tiles take.  No device needed."""
import pytest

from paper_2511_11729_amd import binding as hb

WS = 192 << 20


def plan(B, n_rows, n_mat, K, n_cu=256, ws=WS):
    return hb.dbg_decode_gemm_plan(B, n_rows, n_mat, K, n_cu, ws)


@pytest.mark.parametrize("B,fm", [(33, 1), (64, 1), (65, 2), (128, 2), (129, 3), (192, 3), (193, 4), (256, 4), (257, 4), (600, 4)])
def test_tile_height_follows_the_batch(B, fm):
    p = plan(B, 4096, 1, 4096)
    assert p["FM"] == fm
    assert p["Mpad"] == p["tiles_m"] * 64 * fm and p["Mpad"] >= B > p["Mpad"] - 64 * fm


@pytest.mark.parametrize("B,n_rows,n_mat,K", [(192, 6144, 1, 4096), (192, 4096, 1, 14336), (256, 11008, 2, 4096), (100, 688, 2, 256),
                                              (70, 3584, 1, 18944), (300, 4608, 1, 3584)])
def test_invariants_of_a_plan(B, n_rows, n_mat, K):
    for n_cu in (256, 230, 128, 26):
        p = plan(B, n_rows, n_mat, K, n_cu)
        steps = -(-K // 32)
        assert p["tiles_n"] == -(-n_rows // 256) * n_mat
        assert 1 <= p["ksplit"] <= max(1, min(32, steps // 8))
        assert p["part_bytes"] == p["ksplit"] * p["Mpad"] * p["tiles_n"] * 256 * 4 <= WS
        assert p["rounds"] == -(-(p["tiles_m"] * p["tiles_n"] * p["ksplit"]) // n_cu)


def test_narrow_outputs_are_cut_along_k_and_wide_ones_are_not():
    narrow = plan(256, 4096, 1, 11008)            # 16 output tiles on 256 compute units
    wide = plan(256, 11008, 2, 4096)              # 86 already
    assert narrow["ksplit"] >= 8 and narrow["rounds"] == 1
    assert wide["ksplit"] <= 3 and wide["rounds"] == 1
    # on a tenth of the chip 16 tiles nearly fill a round: few ranges
    assert plan(256, 4096, 1, 11008, n_cu=26)["ksplit"] <= 4


def test_workspace_caps_the_ranges():
    free = plan(256, 4096, 1, 11008)
    one = 256 * 16 * 256 * 4                       # one partial matrix
    assert plan(256, 4096, 1, 11008, ws=3 * one + 17)["ksplit"] == 3 < free["ksplit"]
    assert plan(256, 4096, 1, 11008, ws=one)["ksplit"] == 1
    assert plan(256, 4096, 1, 11008, ws=one - 1)["ksplit"] == 0     # not even one fits: the step refuses


def test_bad_arguments():
    for args in ((0, 4096, 1, 4096, 256, WS), (64, 0, 1, 4096, 256, WS), (64, 4096, 3, 4096, 256, WS), (64, 4096, 1, 0, 256, WS),
                 (64, 4096, 1, 4096, 0, WS), (64, 4096, 1, 4096, 256, -1)):
        with pytest.raises(hb.HarliError):
            hb.dbg_decode_gemm_plan(*args)
