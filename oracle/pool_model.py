"""Brute-force model of the unified memory pool (TEST INFRASTRUCTURE).

Follows the paper's allocator (Sec. 4.2 two-level chunk/block management,
Sec. 4.4 inference priority through a reserve, Sec. 4.5 small-tensor buddy
pool) with explicit Python sets and linear scans, so the C++ pool can be
compared id for id and byte offset for byte offset over random traces.  Only
tests import this file.

Layout of the slab: [small-tensor pool | chunk 0 | chunk 1 | ...].
  * chunk = n_layers x 2 blocks (Sec. 4.2); a chunk is FREE, KV or TENSOR and
    goes back to FREE when everything in it has been released.
  * KV chunk: block 2*layer+kv holds that layer's K or V; the chunk offers
    pages_per_block = floor(block_bytes / page_bytes) columns; a page id is
    chunk * pages_per_block + slot and addresses the same 16 tokens in every
    layer (the 2-D grid of Sec. 4.2).
  * TENSOR chunk: every tensor takes an integer number of blocks, contiguous.
  * small pool: buddy allocator with a 2 KiB granule (Sec. 4.5), organised as
    arenas of one block each.

Where the paper gives no rule, the policy is fixed as "lowest index first":
  KV page   -> lowest free page id over the existing KV chunks, else the
               lowest FREE chunk becomes KV.  KV may take any FREE chunk.
  TENSOR    -> needs ceil(bytes / block_bytes) blocks.  If that fits in one
               chunk: lowest TENSOR chunk with a long enough free run, lowest
               run start; else the lowest FREE chunk becomes TENSOR.  Larger
               requests take the lowest run of adjacent FREE chunks.  Turning
               a FREE chunk into a TENSOR chunk must leave `kv_reserve_chunks`
               FREE chunks behind (inference has priority), else out-of-memory.
  SMALL     -> bytes < block_bytes, rounded up to granule * 2^k; smallest
               sufficient order first, lowest address within the order; when
               no arena can serve it, one TENSOR block is used instead.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

FREE, KV, TENSOR = 0, 1, 2
CLS_KV_PAGE, CLS_TENSOR, CLS_SMALL, CLS_AUTO = 0, 1, 2, 3


class PoolOOM(Exception):
    pass


class PoolModel:
    def __init__(self, slab_bytes: int, block_bytes: int, n_layers: int, page_tokens: int,
                 kv_row_bytes: int, small_pool_bytes: int, small_granule: int, kv_reserve_chunks: int):
        assert small_pool_bytes % block_bytes == 0
        order = block_bytes // small_granule
        assert order * small_granule == block_bytes and order & (order - 1) == 0
        self.block_bytes, self.n_layers = block_bytes, n_layers
        self.page_bytes = page_tokens * kv_row_bytes
        self._kv_row_bytes = kv_row_bytes
        self.ppb = block_bytes // self.page_bytes
        assert self.ppb >= 1
        self.bpc = 2 * n_layers
        self.chunk_bytes = self.bpc * block_bytes
        self.small_pool_bytes, self.granule = small_pool_bytes, small_granule
        self.n_chunks = (slab_bytes - small_pool_bytes) // self.chunk_bytes
        self.reserve = kv_reserve_chunks
        self.max_order = order.bit_length() - 1
        self.cls = [FREE] * self.n_chunks
        self.kv_used: Dict[int, set] = {}                      # chunk -> used slots
        self.blk_used: Dict[int, List[bool]] = {}              # chunk -> per-block flag
        self.small_free = {(a * block_bytes, self.max_order) for a in range(small_pool_bytes // block_bytes)}
        self.live: Dict[int, Tuple[int, int]] = {}             # offset -> (class actually used, bytes reserved)
        self.small_fallbacks = 0

    # -- helpers ------------------------------------------------------------
    def chunk_base(self, c: int) -> int:
        return self.small_pool_bytes + c * self.chunk_bytes

    def free_chunks(self) -> int:
        return sum(1 for c in self.cls if c == FREE)

    def kv_offset(self, page: int, layer: int, kv: int) -> int:
        c, slot = divmod(page, self.ppb)
        return self.chunk_base(c) + (2 * layer + kv) * self.block_bytes + slot * self.page_bytes

    # -- KV pages -----------------------------------------------------------
    def alloc_page(self) -> int:
        best = None
        for c in range(self.n_chunks):
            if self.cls[c] == KV:
                for s in range(self.ppb):
                    if s not in self.kv_used[c]:
                        best = c * self.ppb + s
                        break
            if best is not None:
                break
        if best is None:
            for c in range(self.n_chunks):
                if self.cls[c] == FREE:
                    self.cls[c] = KV
                    self.kv_used[c] = set()
                    best = c * self.ppb
                    break
        if best is None:
            raise PoolOOM("no chunk for a KV page")
        c, s = divmod(best, self.ppb)
        self.kv_used[c].add(s)
        return best

    def free_page(self, page: int) -> None:
        c, s = divmod(page, self.ppb)
        assert self.cls[c] == KV and s in self.kv_used[c]
        self.kv_used[c].remove(s)
        if not self.kv_used[c]:
            del self.kv_used[c]
            self.cls[c] = FREE

    # -- tensors ------------------------------------------------------------
    def _take_free_chunks(self, start: int, n: int) -> None:
        for c in range(start, start + n):
            self.cls[c] = TENSOR
            self.blk_used[c] = [False] * self.bpc

    def alloc_tensor(self, nbytes: int) -> Tuple[int, int]:
        nblk = max(1, -(-nbytes // self.block_bytes))
        if nblk <= self.bpc:
            for c in range(self.n_chunks):
                if self.cls[c] != TENSOR:
                    continue
                used = self.blk_used[c]
                for b0 in range(self.bpc - nblk + 1):
                    if not any(used[b0:b0 + nblk]):
                        return self._mark(c, b0, nblk)
            if self.free_chunks() - 1 < self.reserve:
                raise PoolOOM("tensor chunk would eat the KV reserve")
            for c in range(self.n_chunks):
                if self.cls[c] == FREE:
                    self._take_free_chunks(c, 1)
                    return self._mark(c, 0, nblk)
            raise PoolOOM("no free chunk")
        need = -(-nblk // self.bpc)
        if self.free_chunks() - need < self.reserve:
            raise PoolOOM("tensor chunks would eat the KV reserve")
        for c in range(self.n_chunks - need + 1):
            if all(self.cls[c + i] == FREE for i in range(need)):
                self._take_free_chunks(c, need)
                return self._mark(c, 0, nblk)
        raise PoolOOM("no run of adjacent free chunks")

    def _mark(self, c: int, b0: int, nblk: int) -> Tuple[int, int]:
        for i in range(nblk):
            cc, bb = c + (b0 + i) // self.bpc, (b0 + i) % self.bpc
            assert not self.blk_used[cc][bb]
            self.blk_used[cc][bb] = True
        off = self.chunk_base(c) + b0 * self.block_bytes
        self.live[off] = (CLS_TENSOR, nblk * self.block_bytes)
        return off, nblk * self.block_bytes

    def _free_tensor(self, off: int, nbytes: int) -> None:
        first = (off - self.small_pool_bytes) // self.block_bytes
        for i in range(nbytes // self.block_bytes):
            cc, bb = divmod(first + i, self.bpc)
            assert self.blk_used[cc][bb]
            self.blk_used[cc][bb] = False
        touched = {(first + i) // self.bpc for i in range(nbytes // self.block_bytes)}
        for cc in touched:
            if not any(self.blk_used[cc]):
                del self.blk_used[cc]
                self.cls[cc] = FREE

    # -- small tensors (buddy) ------------------------------------------------
    def alloc_small(self, nbytes: int) -> Tuple[int, int]:
        order = 0
        while (self.granule << order) < nbytes:
            order += 1
        assert order <= self.max_order
        for o in range(order, self.max_order + 1):
            cands = [off for (off, oo) in self.small_free if oo == o]
            if cands:
                off = min(cands)
                self.small_free.remove((off, o))
                while o > order:                      # split, keep the lower half
                    o -= 1
                    self.small_free.add((off + (self.granule << o), o))
                self.live[off] = (CLS_SMALL, self.granule << order)
                return off, self.granule << order
        got = self.alloc_tensor(self.block_bytes)      # pool exhausted: one general block
        self.small_fallbacks += 1                      # counted only when the block was granted
        return got

    def _free_small(self, off: int, nbytes: int) -> None:
        o = (nbytes // self.granule).bit_length() - 1
        while o < self.max_order:
            buddy = off ^ (self.granule << o)
            if (buddy, o) not in self.small_free:
                break
            self.small_free.remove((buddy, o))
            off = min(off, buddy)
            o += 1
        self.small_free.add((off, o))

    # -- by-size front end ------------------------------------------------------
    def alloc(self, nbytes: int) -> Tuple[int, int]:
        assert nbytes > 0
        return self.alloc_small(nbytes) if nbytes < self.block_bytes else self.alloc_tensor(nbytes)

    def free(self, off: int) -> None:
        cls, nbytes = self.live.pop(off)
        if cls == CLS_SMALL:
            self._free_small(off, nbytes)
        else:
            self._free_tensor(off, nbytes)

    # -- inter-task coordination (Sec. 4.4) -------------------------------------------
    def reserve_chunks_for(self, release_time: float, slo: float, max_bs: int) -> int:
        """Chunks that hold Memory_reserved = (T / SLO) * max_bs * Mem_kv at page granularity: while the finetune
        task takes `release_time` to give memory back, decode runs ceil(release_time / slo) steps and each of at
        most max_bs sequences appends one token per step.  KV memory is handed out in pages of page_tokens tokens,
        so a sequence may need ceil(steps / page_tokens) new pages in that window (a sequence that has just started
        needs its first page for its first token): the reserve is max_bs times that many pages, in whole chunks."""
        import math
        steps = math.ceil(release_time / slo - 1e-12)
        page_tokens = self.page_bytes // self._kv_row_bytes
        pages = max_bs * (-(-steps // page_tokens))
        return -(-pages // self.ppb)

    def kv_row_bytes_(self) -> int:
        return self._kv_row_bytes

    def set_reserve(self, chunks: int) -> None:
        assert chunks >= 0
        self.reserve = chunks

    def pressure(self) -> int:
        """Chunks the finetune task should relinquish now: the shortfall of FREE chunks against the reserve, but
        no more than the TENSOR chunks that exist."""
        short = max(0, self.reserve - self.free_chunks())
        return min(short, sum(1 for c in self.cls if c == TENSOR))

    # -- invariants -----------------------------------------------------------------
    def is_pristine(self) -> bool:
        full = {(a * self.block_bytes, self.max_order) for a in range(self.small_pool_bytes // self.block_bytes)}
        return (all(c == FREE for c in self.cls) and not self.live and self.small_free == full
                and not self.kv_used and not self.blk_used)
