"""Pins for the paged cache, the pool grid and the pool model (CPU only)."""
import json
import os

import numpy as np
import pytest

from oracle import harli_oracle as O
from oracle.pool_model import PoolModel, PoolOOM, FREE, KV, TENSOR
from tests.test_oracle_math import tiny_shapes, rand_weights

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))
MiB = 1 << 20


# ----------------------------------------------------------------------------- geometry vs the paper's constants
def test_paper_constants_llama3_8b():
    # Sec. 4.2: 2 KB per token per layer (one of K or V) for Llama3-8B = 8 KV heads x 128 x 2 B
    row = 8 * 128 * 2
    assert row == GOLD["kv_entry_bytes_llama3_8b"]["value"]
    g = O.PoolGeometry(block_bytes=GOLD["block_bytes"]["value"], n_layers=32, page_tokens=16,
                       kv_row_bytes=row, small_pool_bytes=0, slab_bytes=4 * 128 * MiB)
    assert g.pages_per_block == 64 and g.pages_per_block * 16 == 1024      # a chunk serves ~a thousand tokens
    assert g.chunk_bytes == 32 * GOLD["blocks_per_chunk_factor"]["value"] * 2 * MiB == 128 * MiB
    assert g.n_chunks == 4


def test_non_dividing_page_size_uses_floor():
    # 13B-class: 40 heads x 128 x 2 B = 10240 B per token; 16-token page = 163840 B; 2 MiB / 163840 = 12.8
    g = O.PoolGeometry(2 * MiB, 40, 16, 10240, 0, 3 * 40 * 2 * 2 * MiB)
    assert g.pages_per_block == 12
    assert g.kv_offset(12, 0, 0) == g.chunk_bytes             # page 12 is slot 0 of chunk 1


def test_kv_offset_is_the_2d_grid():
    """Enumerate the grid in memory order: chunk, then (layer, K/V) row, then column."""
    g = O.PoolGeometry(block_bytes=4096, n_layers=3, page_tokens=4, kv_row_bytes=96,
                       small_pool_bytes=8192, slab_bytes=8192 + 5 * 3 * 2 * 4096)
    assert g.pages_per_block == 4096 // 384 == 10
    expect = {}
    cursor = g.small_pool_bytes
    for chunk in range(g.n_chunks):
        for layer in range(3):
            for kv in range(2):
                for slot in range(g.pages_per_block):
                    expect[(chunk * g.pages_per_block + slot, layer, kv)] = cursor + slot * 384
                cursor += 4096
    assert cursor == g.slab_bytes
    for key, off in expect.items():
        assert g.kv_offset(*key) == off
    # pages never overlap
    spans = sorted((off, off + 384) for off in expect.values())
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    # one page id names the same column in every row of its chunk
    assert g.kv_offset(7, 2, 1) - g.kv_offset(7, 0, 0) == 5 * 4096
    # inside a page: [kv head][token slot][head_dim]; 96 B rows = 3 heads x 8 x 4 B
    assert g.head_offset(7, 1, 0, 0, 0, 32) == g.kv_offset(7, 1, 0)
    assert g.head_offset(7, 1, 0, 2, 3, 32) == g.kv_offset(7, 1, 0) + (2 * 4 + 3) * 32
    assert g.head_offset(7, 1, 0, 2, 3, 32) + 32 <= g.kv_offset(7, 1, 0) + g.page_bytes


# ----------------------------------------------------------------------------- paged == contiguous
def _geom(sh, n_layers, n_chunks, block_bytes=4096, elem=4, small=0):
    row = sh.n_kv * sh.head_dim * elem
    return O.PoolGeometry(block_bytes, n_layers, 16, row, small, small + n_chunks * n_layers * 2 * block_bytes)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_paged_equals_contiguous_bit_for_bit(seed):
    rng = np.random.default_rng(100 + seed)
    sh = tiny_shapes(n_kv=2, d=4)
    W = rand_weights(rng, sh)
    geom = _geom(sh, 1, 6, block_bytes=2048, small=2048)       # 512 B pages -> 4 pages per block
    assert geom.pages_per_block == 4
    B = 3
    lens = [5, 31, 16]                                         # 16: the new token opens a fresh page
    n_pages = [(n + 1 + 15) // 16 for n in lens]
    perm = rng.permutation(geom.n_chunks * geom.pages_per_block)[: sum(n_pages)]
    table = np.full((B, max(n_pages)), -1, np.int64)
    it = iter(perm)
    for b in range(B):
        for i in range(n_pages[b]):
            table[b, i] = next(it)
    kv = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    cache = []
    for b, n in enumerate(lens):
        K, V = rng.standard_normal((n, sh.n_kv, sh.head_dim)), rng.standard_normal((n, sh.n_kv, sh.head_dim))
        cache.append((K, V))
        for t in range(n):
            kv.write(table[b], 0, t, K[t], V[t])
    x = rng.standard_normal((B, sh.hidden))
    y_c, new_cache = O.decode_layer_contiguous(x, W, sh, cache)
    y_p = O.decode_layer_paged(x, W, sh, kv, 0, np.array(lens), table)
    assert np.array_equal(y_c, y_p)
    for b, n in enumerate(lens):
        K, V = kv.gather(table[b], 0, n + 1)
        assert np.array_equal(K, new_cache[b][0]) and np.array_equal(V, new_cache[b][1])


def test_page_walk_integer_round_trip():
    sh = tiny_shapes(n_kv=2, d=4)
    geom = _geom(sh, 2, 4, block_bytes=1024)                   # 512 B pages -> 2 per block
    kv = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    rng = np.random.default_rng(7)
    table = rng.permutation(8)[:5]
    n = 5 * 16 - 3
    for layer in range(2):
        for t in range(n):
            code = np.arange(8).reshape(2, 4) + 1000 * t + 100000 * layer
            kv.write(table, layer, t, code, -code)
    for layer in range(2):
        K, V = kv.gather(table, layer, n)
        for t in range(n):
            code = np.arange(8).reshape(2, 4) + 1000 * t + 100000 * layer
            assert np.array_equal(K[t], code) and np.array_equal(V[t], -code)
    # every written element sits where the address function says, nothing else was touched
    touched = np.flatnonzero(kv.slab)
    want = set()
    for layer in range(2):
        for t in range(n):
            for which in (0, 1):
                for head in range(2):
                    off = geom.head_offset(int(table[t // 16]), layer, which, head, t % 16, 16) // 4
                    want.update(range(off, off + 4))
    # code 0 (t=0, layer=0, first element of K) is a legitimate zero
    assert set(touched.tolist()) <= want and len(want) - len(touched) <= 2


def test_multi_layer_model_is_a_stack_of_layers():
    rng = np.random.default_rng(21)
    sh = tiny_shapes(n_kv=2, d=4)
    layers = [rand_weights(rng, sh) for _ in range(3)]
    geom = _geom(sh, 3, 2, block_bytes=2048)
    kv = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    lens = np.array([3, 17])
    table = np.array([[5, -1], [2, 7]])
    for l in range(3):
        for b in range(2):
            for t in range(lens[b]):
                kv.write(table[b], l, t, rng.standard_normal((2, 4)), rng.standard_normal((2, 4)))
    x = rng.standard_normal((2, sh.hidden))
    kv2 = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim, slab=kv.slab.copy())
    out = O.decode_model_paged(x, layers, None, sh, kv, lens, table)
    ref = x
    for l in range(3):
        ref = O.decode_layer_paged(ref, layers[l], sh, kv2, l, lens, table)
    assert np.array_equal(out, ref) and np.array_equal(kv.slab, kv2.slab)
    # with an embedding and an output layer: gather, final norm, matmul, argmax
    extras = dict(emb=rng.standard_normal((11, sh.hidden)), gf=np.ones(sh.hidden), wlm=rng.standard_normal((11, sh.hidden)))
    kv3 = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim, slab=kv2.slab.copy())
    hid, logits, nxt = O.decode_model_paged(np.array([4, 9]), layers, extras, sh, kv3, lens + 1, table)
    assert logits.shape == (2, 11) and np.array_equal(nxt, logits.argmax(-1))
    assert np.allclose(logits, O.rmsnorm(hid, extras["gf"], sh.rms_eps) @ extras["wlm"].T)


def test_full_model_embedding_gather_final_norm_and_output_layer():
    """Pins the three steps around the layer stack (Sec. 2.1: embedding, layers, output layer) to values worked out by
    hand: the row of the table a token id selects, the final norm with gains that are not one, the output product
    written as explicit sums, and the lowest index on an argmax tie."""
    sh = tiny_shapes(n_kv=2, d=4)
    H = sh.hidden
    geom = _geom(sh, 1, 2, block_bytes=2048)
    kv = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    V = 11
    emb = np.arange(V, dtype=np.float64)[:, None] * np.ones((1, H))     # row i is the constant i
    gf = 1.0 + 0.1 * np.arange(H)
    wlm = np.zeros((V, H))
    wlm[3, 0], wlm[7, 0], wlm[5, 1] = 2.0, 2.0, 1.0                     # rows 3 and 7 tie
    tokens = np.array([4, 9])
    # no layers: the hidden state is the gathered row itself
    hid, logits, nxt = O.decode_model_paged(tokens, [], dict(emb=emb, gf=gf, wlm=wlm), sh, kv, np.array([0, 0]),
                                            np.array([[0], [1]]))
    assert np.array_equal(hid, np.stack([np.full(H, 4.0), np.full(H, 9.0)]))
    for b, c in enumerate((4.0, 9.0)):
        rho = 1.0 / np.sqrt(c * c + sh.rms_eps)                         # mean of squares of a constant row
        want = np.zeros(V)
        for v in range(V):
            for j in range(H):
                want[v] += c * rho * gf[j] * wlm[v, j]
        assert np.allclose(logits[b], want, rtol=1e-13, atol=0)
        assert logits[b, 3] == logits[b, 7] > logits[b, 5] and nxt[b] == 3
    # with layers: token ids give what the gathered rows give when passed as hidden states
    rng = np.random.default_rng(5)
    layers = [rand_weights(rng, sh)]
    emb2 = rng.standard_normal((V, H))
    lens, table = np.array([0, 0]), np.array([[0], [1]])
    kv_a = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    kv_b = O.PagedKV(geom, 4, sh.n_kv, sh.head_dim)
    hid_t, _, _ = O.decode_model_paged(tokens, layers, dict(emb=emb2, gf=gf, wlm=wlm), sh, kv_a, lens, table)
    x_rows = np.stack([emb2[4], emb2[9]])
    hid_x = O.decode_model_paged(x_rows, layers, None, sh, kv_b, lens, table)
    assert np.array_equal(hid_t, hid_x) and np.array_equal(kv_a.slab, kv_b.slab)
    swapped = O.decode_model_paged(np.stack([emb2[9], emb2[4]]), layers, None, sh,
                                   O.PagedKV(geom, 4, sh.n_kv, sh.head_dim), lens, table)
    assert not np.allclose(hid_t, swapped)


# ----------------------------------------------------------------------------- pool model
def mk_pool(n_chunks=6, n_layers=2, block=8192, small_blocks=2, reserve=1, row=256):
    small = small_blocks * block
    return PoolModel(small + n_chunks * 2 * n_layers * block + 100, block, n_layers, 16, row, small, 2048, reserve)


def test_buddy_textbook_sequence():
    p = mk_pool(small_blocks=1)                      # one 8 KiB arena = 4 granules of 2 KiB
    a = p.alloc_small(100)
    b = p.alloc_small(2048)
    c = p.alloc_small(2049)                          # rounds to 4 KiB
    assert (a, b, c) == ((0, 2048), (2048, 2048), (4096, 4096))
    p.free(a[0])
    d = p.alloc_small(3000)                          # needs 4 KiB: none free -> falls back to a tensor block
    assert d[0] >= p.small_pool_bytes and p.small_fallbacks == 1
    p.free(b[0])                                     # a and b coalesce into a 4 KiB buddy
    e = p.alloc_small(4096)
    assert e == (0, 4096)
    for off in (c[0], d[0], e[0]):
        p.free(off)
    assert p.is_pristine()


def test_kv_pages_lowest_id_first_and_chunk_return():
    p = mk_pool(row=256)                             # page = 4096 B, 2 pages per block
    assert p.ppb == 2
    ids = [p.alloc_page() for _ in range(5)]
    assert ids == [0, 1, 2, 3, 4]
    assert p.cls[:3] == [KV, KV, KV]
    p.free_page(2)
    p.free_page(3)
    assert p.cls[1] == FREE                          # all columns of chunk 1 free -> back to the pool
    p.free_page(0)
    assert p.alloc_page() == 0                       # lowest id first
    assert p.alloc_page() == 5                       # existing KV chunks are filled before a new chunk is taken
    assert p.alloc_page() == 2                       # then chunk 1 is taken again as the lowest free chunk
    assert p.kv_offset(2, 1, 1) == p.small_pool_bytes + p.chunk_bytes + 3 * p.block_bytes


def test_tensor_blocks_first_fit_reserve_and_multi_chunk():
    p = mk_pool(n_chunks=6, n_layers=2, reserve=1)   # 4 blocks per chunk
    a = p.alloc_tensor(8192 * 3)                     # chunk 0 blocks 0..2
    b = p.alloc_tensor(8192 * 2)                     # does not fit chunk 0 -> chunk 1 blocks 0..1
    c = p.alloc_tensor(8192)                         # chunk 0 block 3
    base = p.small_pool_bytes
    assert a == (base, 3 * 8192) and b == (base + p.chunk_bytes, 2 * 8192) and c == (base + 3 * 8192, 8192)
    big = p.alloc_tensor(p.chunk_bytes * 2 + 1)      # 9 blocks -> 3 adjacent free chunks: 2,3,4
    assert big[0] == base + 2 * p.chunk_bytes and big[1] == 9 * 8192
    assert p.cls == [TENSOR, TENSOR, TENSOR, TENSOR, TENSOR, FREE]
    with pytest.raises(PoolOOM):                     # the last free chunk is the KV reserve
        p.alloc_tensor(8192 * 4)
    assert p.alloc_page() == 5 * p.ppb               # KV may use it
    d = p.alloc_tensor(8192 * 3)                     # tail of chunk 4 (blocks 1..3) is still usable
    assert d[0] == base + 4 * p.chunk_bytes + 8192
    for off in (a[0], b[0], c[0], big[0], d[0]):
        p.free(off)
    p.free_page(5 * p.ppb)
    assert p.is_pristine()


@pytest.mark.parametrize("seed", range(4))
def test_random_trace_never_overlaps_and_returns_to_pristine(seed):
    rng = np.random.default_rng(seed)
    p = mk_pool(n_chunks=8, n_layers=2, block=8192, small_blocks=2, reserve=1, row=128)
    live, pages = {}, []
    for _ in range(600):
        r = rng.random()
        try:
            if r < 0.3:
                pages.append(p.alloc_page())
            elif r < 0.6:
                n = int(rng.choice([1, 100, 2048, 3000, 5000, 8191, 8192, 20000, 40000, 70000]))
                off, sz = p.alloc(n)
                assert sz >= n
                live[off] = sz
            elif r < 0.8 and pages:
                p.free_page(pages.pop(int(rng.integers(len(pages)))))
            elif live:
                off = list(live)[int(rng.integers(len(live)))]
                p.free(off)
                del live[off]
        except PoolOOM:
            pass
        spans = sorted((o, o + s) for o, s in live.items())
        for pg in pages:
            for l in range(2):
                for kv in range(2):
                    o = p.kv_offset(pg, l, kv)
                    spans.append((o, o + p.page_bytes))
        spans.sort()
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        assert len(set(pages)) == len(pages)
    for pg in pages:
        p.free_page(pg)
    for off in list(live):
        p.free(off)
    assert p.is_pristine()


# ---- inter-task memory coordination (Sec. 4.4): the reserve formula and the back-pressure count ----

def _coord_model(n_chunks=12, n_layers=2, reserve=0):
    from oracle.pool_model import PoolModel
    block = 64 << 10
    return PoolModel(n_chunks * n_layers * 2 * block, block, n_layers, 16, 512, 0, 2048, reserve)


def test_reserve_formula_hand_values():
    """Memory_reserved = (T/SLO) * max_bs * Mem_kv at page granularity, in whole chunks.  Geometry: 64 KiB blocks,
    512 B rows, 16-token pages -> 8 pages per chunk."""
    m = _coord_model()
    assert m.ppb == 8
    # release 100 ms, SLO 50 ms: two decode steps, at most one new page per sequence; 64 sequences -> 64 pages
    assert m.reserve_chunks_for(100.0, 50.0, 64) == 8
    assert m.reserve_chunks_for(100.0, 50.0, 65) == 9
    assert m.reserve_chunks_for(25.0, 50.0, 1) == 1            # half a step still needs the token's page
    assert m.reserve_chunks_for(0.0, 50.0, 256) == 0
    assert m.reserve_chunks_for(80.0, 50.0, 256) == 32
    # a release lasting 20 steps can cross two page boundaries per sequence: 8 sequences -> 16 pages -> 2 chunks
    assert m.reserve_chunks_for(1000.0, 50.0, 8) == 2
    assert m.reserve_chunks_for(800.0, 50.0, 8) == 1           # 16 steps: one page each


def test_pressure_counts_the_shortfall_against_the_reserve():
    m = _coord_model(n_chunks=6, reserve=2)
    t = [m.alloc_tensor(m.chunk_bytes) for _ in range(4)]      # four TENSOR chunks, two FREE left = the reserve
    assert m.free_chunks() == 2 and m.pressure() == 0
    import pytest
    from oracle.pool_model import PoolOOM
    with pytest.raises(PoolOOM):
        m.alloc_tensor(m.chunk_bytes)                          # would eat the reserve
    pages = [m.alloc_page() for _ in range(m.ppb + 1)]         # decode grows into the reserve: two KV chunks
    assert m.free_chunks() == 0 and m.pressure() == 2
    m.free(t[0][0])
    assert m.pressure() == 1
    m.set_reserve(5)
    assert m.pressure() == 3                                   # never more than the TENSOR chunks that exist
    for pg in pages:
        m.free_page(pg)
    m.set_reserve(2)
    assert m.pressure() == 0
