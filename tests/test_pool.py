"""The C++ pool against the brute-force pool model: ids and offsets must match exactly (CPU only).

The slab address is never dereferenced by the pool, so a fake base pointer is enough.
"""
import numpy as np
import pytest

from oracle.pool_model import PoolModel, PoolOOM
from paper_2511_11729_amd import binding as hb

BASE = 0x7000_0000_0000


def make(n_chunks=8, n_layers=2, block=8192, small_blocks=2, reserve=1, row=128, extra=100):
    small = small_blocks * block
    slab = small + n_chunks * 2 * n_layers * block + extra
    model = PoolModel(slab, block, n_layers, 16, row, small, 2048, reserve)
    pool = hb.Pool(BASE, slab, block_bytes=block, n_layers=n_layers, page_tokens=16, kv_row_bytes=row,
                   small_pool_bytes=small, small_granule=2048, kv_reserve_chunks=reserve)
    return model, pool


@pytest.mark.parametrize("seed", range(6))
def test_random_trace_matches_model(seed):
    rng = np.random.default_rng(seed)
    model, pool = make(n_chunks=int(rng.integers(3, 12)), n_layers=int(rng.integers(1, 4)),
                       small_blocks=int(rng.integers(0, 3)), reserve=int(rng.integers(0, 3)),
                       row=int(rng.choice([64, 128, 160, 512])))
    st = pool.stats()
    assert st.n_chunks == model.n_chunks and st.pages_per_block == model.ppb and st.blocks_per_chunk == model.bpc
    live, pages = {}, []
    sizes = [1, 100, 2048, 2049, 3000, 5000, 8191, 8192, 8193, 20000, 40000, 70000, 150000]
    for step in range(1500):
        r = rng.random()
        if r < 0.3:
            try:
                want = model.alloc_page()
            except PoolOOM:
                with pytest.raises(hb.HarliError) as e:
                    pool.alloc(hb.CLS_KV_PAGE)
                assert e.value.status == hb.HARLI_ERR_OOM
                continue
            got = pool.alloc(hb.CLS_KV_PAGE)
            assert got.page == want, step
            pages.append(want)
        elif r < 0.6:
            n = int(rng.choice(sizes))
            if n < model.block_bytes and model.small_pool_bytes == 0 and False:
                continue
            try:
                off, sz = model.alloc(n)
            except PoolOOM:
                with pytest.raises(hb.HarliError) as e:
                    pool.alloc(hb.CLS_AUTO, n)
                assert e.value.status == hb.HARLI_ERR_OOM
                continue
            a = pool.alloc(hb.CLS_AUTO, n)
            assert (a.offset, a.bytes) == (off, sz), step
            assert a.ptr == BASE + off
            live[off] = a
        elif r < 0.8 and pages:
            pg = pages.pop(int(rng.integers(len(pages))))
            model.free_page(pg)
            pool.free_pages([pg])
        elif live:
            off = list(live)[int(rng.integers(len(live)))]
            model.free(off)
            pool.free(live.pop(off))
        st = pool.stats()
        assert st.free_chunks == model.free_chunks()
        assert st.kv_pages_live == len(pages)
        assert st.small_fallbacks == model.small_fallbacks
    for pg in pages:
        assert pool.kv_addr(pg, model.n_layers - 1, 1) == model.kv_offset(pg, model.n_layers - 1, 1)
    pool.free_pages(pages)
    for pg in pages:
        model.free_page(pg)
    for off, a in live.items():
        model.free(off)
        pool.free(a)
    assert model.is_pristine()
    st = pool.stats()
    assert st.free_chunks == st.n_chunks and st.kv_pages_live == 0 and st.tensor_blocks_live == 0
    assert st.small_bytes_live == 0 and st.reserved_bytes_live == 0 and st.requested_bytes_live == 0
    # a pristine pool hands out the same first ids again
    assert pool.alloc(hb.CLS_KV_PAGE).page == 0


def test_kv_addr_matches_model_everywhere():
    model, pool = make(n_chunks=5, n_layers=3, block=8192, row=160)      # 2560 B pages: 3 per block, slack at the tail
    assert model.ppb == 3
    for page in range(model.n_chunks * model.ppb):
        for layer in range(3):
            for kv in range(2):
                assert pool.kv_addr(page, layer, kv) == model.kv_offset(page, layer, kv)
    with pytest.raises(hb.HarliError):
        pool.kv_addr(model.n_chunks * model.ppb, 0, 0)
    with pytest.raises(hb.HarliError):
        pool.kv_addr(0, 3, 0)


def test_error_paths():
    model, pool = make()
    a = pool.alloc(hb.CLS_AUTO, 5000)
    pool.free(a)
    with pytest.raises(hb.HarliError) as e:
        pool.free(a)                                  # double free
    assert e.value.status == hb.HARLI_ERR_INVALID
    with pytest.raises(hb.HarliError):
        pool.free_pages([3])                          # never allocated
    with pytest.raises(hb.HarliError):
        pool.alloc(hb.CLS_SMALL, 8192)                # SMALL must be below one block
    with pytest.raises(hb.HarliError):
        pool.alloc(hb.CLS_TENSOR, 0)
    ids = pool.alloc_pages(3)
    with pytest.raises(hb.HarliError):
        pool.free_pages([ids[0], ids[0]])
    pool.free_pages(ids)
    # all-or-nothing batch allocation
    total = pool.stats().n_chunks * pool.stats().pages_per_block
    with pytest.raises(hb.HarliError) as e:
        pool.alloc_pages(total + 1)
    assert e.value.status == hb.HARLI_ERR_OOM
    assert pool.stats().kv_pages_live == 0 and pool.stats().free_chunks == pool.stats().n_chunks


def test_reserve_keeps_chunks_for_kv():
    model, pool = make(n_chunks=4, n_layers=1, block=8192, small_blocks=0, reserve=2)
    pool.alloc(hb.CLS_TENSOR, 8192 * 2)
    pool.alloc(hb.CLS_TENSOR, 8192 * 2)
    with pytest.raises(hb.HarliError) as e:
        pool.alloc(hb.CLS_TENSOR, 8192)               # would leave only one free chunk
    assert e.value.status == hb.HARLI_ERR_OOM
    assert pool.alloc(hb.CLS_KV_PAGE).page == 2 * pool.stats().pages_per_block   # KV may dip into the reserve
