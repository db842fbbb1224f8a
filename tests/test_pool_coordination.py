"""Inter-task memory coordination (Sec. 4.4): the library's reserve formula, reserve update and back-pressure
count against the pool model, and a replay of the paper's load phases (light 8 -> heavy 42 -> medium 24
sequences, Sec. 8.5) in which decode and finetune allocate from the same pool.  CPU only."""
import numpy as np
import pytest

from oracle.pool_model import PoolModel, PoolOOM
from paper_2511_11729_amd import binding as hb

BASE = 0x7000_0000_0000


def make(n_chunks, n_layers=2, block=64 << 10, row=512, reserve=0):
    slab = n_chunks * 2 * n_layers * block
    model = PoolModel(slab, block, n_layers, 16, row, 0, 2048, reserve)
    pool = hb.Pool(BASE, slab, block_bytes=block, n_layers=n_layers, page_tokens=16, kv_row_bytes=row,
                   small_pool_bytes=0, small_granule=2048, kv_reserve_chunks=reserve)
    return model, pool


@pytest.mark.parametrize("seed", range(4))
def test_reserve_formula_matches_the_model(seed):
    rng = np.random.default_rng(seed)
    model, pool = make(6, n_layers=int(rng.integers(1, 5)), row=int(rng.choice([128, 512, 640, 2048])))
    for _ in range(300):
        T = float(rng.uniform(0, 500))
        slo = float(rng.choice([40.0, 50.0, 80.0, 1.25]))
        bs = int(rng.integers(1, 257))
        assert pool.reserve_chunks_for(T, slo, bs) == model.reserve_chunks_for(T, slo, bs)
    assert pool.reserve_chunks_for(100.0, 50.0, 64) == model.reserve_chunks_for(100.0, 50.0, 64)
    assert pool.reserve_chunks_for(1000.0, 50.0, 8) == model.reserve_chunks_for(1000.0, 50.0, 8)
    for bad in [(-1.0, 50.0, 8), (10.0, 0.0, 8), (10.0, 50.0, 0), (float("nan"), 50.0, 8)]:
        with pytest.raises(hb.HarliError):
            pool.reserve_chunks_for(*bad)
    with pytest.raises(hb.HarliError):
        pool.set_reserve(-1)


def test_load_phases_replay():
    """Decode: `bs` sequences, each appending one token per step (a new page every 16 steps), sequences finish after
    a seeded number of tokens and are replaced.  Finetune: every step tries to take three units' activations (three
    chunks' worth each) and gives each back seven steps later; when the pool reports pressure it releases its
    oldest units at once and skips the step.  Both sides must agree on every id, offset, failure and pressure reading."""
    n_chunks = 100
    model, pool = make(n_chunks)
    # reserve from the formula: releasing takes two decode steps' time, up to 48 sequences
    reserve = pool.reserve_chunks_for(100.0, 50.0, 48)
    assert reserve == model.reserve_chunks_for(100.0, 50.0, 48) == 6
    pool.set_reserve(reserve)
    model.set_reserve(reserve)
    rng = np.random.default_rng(11)
    unit_bytes = 3 * model.chunk_bytes
    seqs = []                  # per sequence: [tokens so far, length at which it ends, pages]
    units = []                 # (age, offset, alloc)
    stats = {"ft_ok": 0, "ft_oom": 0, "ft_yield": 0, "kv_fail": 0, "max_kv_chunks": 0}
    phases = [(8, 150), (42, 260), (24, 150)]
    log = []
    ok_per_step = []
    for bs, steps in phases:
        for _ in range(steps):
            # ---- decode step
            while len(seqs) > bs:
                s = seqs.pop()
                for pg in s[2]:
                    model.free_page(pg)
                pool.free_pages(s[2])
            while len(seqs) < bs:
                seqs.append([0, int(rng.integers(64, 400)), []])
            for s in list(seqs):
                if s[0] % 16 == 0:
                    try:
                        want = model.alloc_page()
                    except PoolOOM:
                        stats["kv_fail"] += 1
                        with pytest.raises(hb.HarliError):
                            pool.alloc(hb.CLS_KV_PAGE)
                        continue
                    got = pool.alloc(hb.CLS_KV_PAGE)
                    assert got.page == want
                    s[2].append(want)
                s[0] += 1
                if s[0] >= s[1]:
                    for pg in s[2]:
                        model.free_page(pg)
                    pool.free_pages(s[2])
                    seqs.remove(s)
            # ---- finetune step
            units = [(age + 1, off, a) for age, off, a in units]
            for age, off, a in [u for u in units if u[0] >= 7]:
                model.free(off)
                pool.free(a)
            units = [u for u in units if u[0] < 7]
            pm, pp = model.pressure(), pool.pressure()
            assert pm == pp
            if pm > 0:
                stats["ft_yield"] += 1
                for _ in range(min(len(units), -(-pm // 3))):      # give the oldest units back at once
                    age, off, a = units.pop(0)
                    model.free(off)
                    pool.free(a)
            else:
                for _ in range(3):
                    try:
                        off, sz = model.alloc_tensor(unit_bytes)
                    except PoolOOM:
                        stats["ft_oom"] += 1
                        with pytest.raises(hb.HarliError) as e:
                            pool.alloc(hb.CLS_TENSOR, unit_bytes)
                        assert e.value.status == hb.HARLI_ERR_OOM
                    else:
                        a = pool.alloc(hb.CLS_TENSOR, unit_bytes)
                        assert (a.offset, a.bytes) == (off, sz)
                        units.append((0, off, a))
                        stats["ft_ok"] += 1
            ok_per_step.append(stats["ft_ok"])
            st = pool.stats()
            assert st.free_chunks == model.free_chunks()
            stats["max_kv_chunks"] = max(stats["max_kv_chunks"], st.kv_chunks)
        log.append((bs, dict(stats), pool.stats().kv_chunks))
    # inference never failed: the reserve and the back-pressure kept room for it through the heavy phase
    assert stats["kv_fail"] == 0
    light, heavy, medium = log
    assert heavy[2] > light[2]                                          # decode's footprint grew in the heavy phase
    squeezed = lambda a, b: (b["ft_oom"] + b["ft_yield"]) - (a["ft_oom"] + a["ft_yield"])
    zero = {"ft_oom": 0, "ft_yield": 0, "ft_ok": 0}
    assert squeezed(zero, light[1]) == 0                                # room for both in the light phase
    assert squeezed(light[1], heavy[1]) > 0                             # finetune was squeezed in the heavy phase
    # ... and recovers as the heavy phase's sequences finish and their chunks come back: more units are admitted in
    # the last 50 steps of the medium phase than in the last 50 of the heavy one
    end_heavy, end_medium = 150 + 260, 150 + 260 + 150
    assert medium[2] < heavy[1]["max_kv_chunks"]
    assert ok_per_step[end_medium - 1] - ok_per_step[end_medium - 51] > ok_per_step[end_heavy - 1] - ok_per_step[end_heavy - 51]
    # wind down: everything returns, the pool is pristine again
    for s in seqs:
        for pg in s[2]:
            model.free_page(pg)
        pool.free_pages(s[2])
    for age, off, a in units:
        model.free(off)
        pool.free(a)
    assert model.is_pristine()
    st = pool.stats()
    assert st.free_chunks == st.n_chunks and st.kv_pages_live == 0 and st.tensor_blocks_live == 0
    print("load phases:", log)


def test_pressure_matches_the_model_when_decode_eats_the_reserve():
    model, pool = make(6, reserve=2)
    held = []
    for _ in range(4):
        off, sz = model.alloc_tensor(model.chunk_bytes)
        a = pool.alloc(hb.CLS_TENSOR, model.chunk_bytes)
        assert (a.offset, a.bytes) == (off, sz)
        held.append((off, a))
    assert pool.pressure() == model.pressure() == 0
    with pytest.raises(hb.HarliError) as e:
        pool.alloc(hb.CLS_TENSOR, model.chunk_bytes)
    assert e.value.status == hb.HARLI_ERR_OOM
    pages = []
    for _ in range(model.ppb + 1):                     # two KV chunks: the whole reserve
        want = model.alloc_page()
        assert pool.alloc(hb.CLS_KV_PAGE).page == want
        pages.append(want)
    assert pool.pressure() == model.pressure() == 2
    off, a = held.pop(0)
    model.free(off)
    pool.free(a)
    assert pool.pressure() == model.pressure() == 1
    pool.set_reserve(5)
    model.set_reserve(5)
    assert pool.pressure() == model.pressure() == 3    # capped by the TENSOR chunks that exist
    pool.set_reserve(0)
    model.set_reserve(0)
    assert pool.pressure() == model.pressure() == 0
    off2, sz2 = model.alloc_tensor(model.chunk_bytes)  # with no reserve the freed chunk can be taken again
    a2 = pool.alloc(hb.CLS_TENSOR, model.chunk_bytes)
    assert (a2.offset, a2.bytes) == (off2, sz2)
