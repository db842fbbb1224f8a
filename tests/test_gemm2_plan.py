"""Launch grid of the finetune unit's weight GEMM (host logic, no GPU): with the workgroup-to-tile rule its header
states every tile of the output is computed exactly once, the workgroups an XCD runs together cover a compact block of
tiles, and the cost counts rounds over the compute units of the stream's partition (Harli Sec. 6.2: the finetune task
runs on a share of the compute units)."""
import itertools

import pytest

from paper_2511_11729_amd import binding as hb


def tiles_of(plan, M, tiles_n, tile_rows):
    GM, GN, total, chunk = plan["GM"], plan["GN"], plan["total"], plan["chunk"]
    nbn = -(-tiles_n // GN)
    cover = {}
    for w in range(plan["grid"]):
        slot = (w & 7) * chunk + (w >> 3)
        if slot >= total:
            continue
        blk, within = divmod(slot, GM * GN)
        bm, bn = divmod(blk, nbn)
        tm, tn = bm * GM + within // GN, bn * GN + within % GN
        if tm * tile_rows >= M or tn >= tiles_n:
            continue
        cover.setdefault((tm, tn), []).append(w)
    return cover


SHAPES = [(2048, 16), (2048, 48), (2048, 86), (2048, 43), (300, 3), (129, 1), (4096, 172), (1000, 7), (64, 5)]


@pytest.mark.parametrize("M,tiles_n", SHAPES)
@pytest.mark.parametrize("tile_rows", [128, 256])
@pytest.mark.parametrize("n_cu", [256, 230, 179, 7])
def test_every_tile_is_computed_once(M, tiles_n, tile_rows, n_cu):
    p = hb.dbg_gemm2_plan(M, tiles_n, tile_rows, n_cu)
    tiles_m = -(-M // tile_rows)
    cover = tiles_of(p, M, tiles_n, tile_rows)
    assert set(cover) == set(itertools.product(range(tiles_m), range(tiles_n)))
    assert all(len(ws) == 1 for ws in cover.values())
    assert p["grid"] == p["chunk"] * 8 and p["rounds"] == -(-tiles_m * tiles_n // n_cu)
    # the 32 workgroups an XCD runs at a time (consecutive slots of its chunk) stay inside one or two blocks of tiles
    if p["total"] >= 8 * 32 and p["GM"] * p["GN"] == 32:
        for x in range(8):
            first = [(x * p["chunk"] + i) // 32 for i in range(32)]
            assert len(set(first)) <= 2


def test_bad_arguments():
    with pytest.raises(hb.HarliError):
        hb.dbg_gemm2_plan(2048, 16, 100, 230)
    with pytest.raises(hb.HarliError):
        hb.dbg_gemm2_plan(2048, 16, 128, 0)
