"""Device-side set-up shared by bench.py and the scheduler profiling: one workload's layer, its paged KV cache
and finetune buffers in a unified pool, and the two calls the co-location runs issue.  Argument marshalling and
buffer ownership only -- every step of the path runs in libharli's kernels."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from . import binding as hb

DEV = "cuda:0"


def dev_bf16(a: np.ndarray):
    return torch.from_numpy(wl.bf16_bits(a).view(np.int16).reshape(a.shape)).to(DEV).view(torch.bfloat16)


def dev_f32(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


class LayerHarness:
    """Config-1-style single layer: decode batch with a paged cache + LoRA finetune unit, one pool for both.

    decode_capacity: (max batch, max cached tokens per sequence) the context and the page tables are sized for;
    the cache is zero-filled beyond the workload's own seeded K/V (the values do not change the traffic)."""

    def __init__(self, w: wl.Workload, *, in_flight: int = 8, decode_capacity=None, fill_kv: bool = True):
        self.w = w
        m, ft, lora = w.model, w.finetune, w.lora
        self.m, self.ft, self.lora = m, ft, lora
        T = ft.tokens
        self.T = T
        self.W_np = wl.make_layer_weights(w, 0)
        self.lora_np = wl.make_lora(w, 0)
        x_np, kv_len, kv_np = wl.make_decode_inputs(w)
        self.X_np, _ = wl.make_finetune_inputs(w)
        self.kv_len = kv_len
        B = len(kv_len)
        self.B = B
        P = 16
        cap_b, cap_n = decode_capacity or (B, int(kv_len.max()) + 1)
        cap_b, cap_n = max(cap_b, B), max(cap_n, int(kv_len.max()) + 1)
        self.cap_b, self.cap_n = cap_b, cap_n
        pages_per_seq = (cap_n + P - 1) // P + 1
        total_pages = cap_b * pages_per_seq
        block = 2 << 20
        chunk = m.n_layers * 2 * block
        ppb = block // (P * m.kv_row_bytes)
        act = (T * m.hidden * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6)
        self.in_flight = in_flight
        # every byte the library keeps (the decode instance's weight copy, the finetune instance's two, both workspaces)
        # comes from the pool as well: one pool for all tensors of both tasks (Sec. 4.2)
        lib_bytes = 6 * m.layer_params + 3 * act + (128 << 20)
        if cap_b >= 17:                                  # the partial tiles of the decode GEMMs above 32 sequences (at most 192 MiB)
            lib_bytes += 192 << 20
        n_chunks = -(-total_pages // ppb) + in_flight * (act // chunk + 2) + lib_bytes // chunk + 8
        small = 64 << 20
        self.slab_bytes = small + n_chunks * chunk
        self.slab = torch.zeros(self.slab_bytes, dtype=torch.uint8, device=DEV)
        self.pool = hb.Pool(self.slab, self.slab_bytes, block_bytes=block, n_layers=m.n_layers, kv_row_bytes=m.kv_row_bytes,
                            small_pool_bytes=small, kv_reserve_chunks=2)
        # KV reserve from the coordination formula (Sec. 4.4): a finetune unit gives its activations back within about
        # two unit times (6 ms); the decode QoS target of this single layer is 40 ms / 32
        self.pool.set_reserve(self.pool.reserve_chunks_for(6.0, 40.0 / 32.0, cap_b))
        ids = np.array(self.pool.alloc_pages(total_pages), np.int64)[wl.page_order(w, total_pages)]
        self.max_pages = pages_per_seq
        table = ids.reshape(cap_b, pages_per_seq).astype(np.int32)
        self.table = table
        if fill_kv:
            img = np.zeros(self.slab_bytes // 2, np.uint16)
            d = m.head_dim
            for b in range(B):
                Kc, Vc = kv_np[0][b]
                for which, Tn in ((0, Kc), (1, Vc)):
                    enc = wl.bf16_bits(Tn).reshape(Tn.shape)
                    n = Tn.shape[0]
                    for lp in range((n + P - 1) // P):
                        t0, t1 = lp * P, min(n, lp * P + P)
                        base = self.pool.kv_addr(int(table[b, lp]), 0, which) // 2
                        for c in range(m.n_kv):
                            off = base + c * P * d
                            img[off: off + (t1 - t0) * d] = enc[t0:t1, c, :].reshape(-1)
            self.slab.copy_(torch.from_numpy(img.view(np.uint8)))
            del img
        layer = {n: dev_bf16(self.W_np[n]) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
        layer["g1"], layer["g2"] = dev_f32(self.W_np["g1"]), dev_f32(self.W_np["g2"])
        for bn in ("bq", "bk", "bv"):
            if bn in self.W_np:
                layer[bn] = dev_f32(self.W_np[bn])
        self.layer = layer
        self.ctx = hb.Context(self.pool, n_layers=1, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv, head_dim=m.head_dim,
                              ffn=m.ffn, rms_eps=m.rms_eps, rope_base=m.rope_base, dtype=hb.HARLI_BF16, max_batch=cap_b,
                              max_seq_len=cap_n + 8, max_ft_tokens=T, layers=[layer], memory_in_pool=True)
        self.A_dev = {p: dev_bf16(a) for p, (a, b) in self.lora_np.items()}
        self.B_dev = {p: dev_bf16(b) for p, (a, b) in self.lora_np.items()}
        self.ctx.lora_attach(lora.rank, lora.alpha, lora.targets, [self.A_dev], [self.B_dev])
        self.table_dev = torch.from_numpy(table).to(DEV)
        self.kv_len_dev = torch.from_numpy(kv_len.astype(np.int32)).to(DEV)
        xs = np.zeros((cap_b, m.hidden), np.float32)
        xs[:B] = x_np
        if cap_b > B:
            xs[B:] = np.resize(x_np, (cap_b - B, m.hidden))
        self.x_dev = dev_f32(xs)
        self.y_dev = torch.empty(cap_b, m.hidden, dtype=torch.float32, device=DEV)
        self.X_dev = dev_f32(self.X_np.reshape(T, m.hidden))
        self.Y_dev = torch.empty(T, m.hidden, dtype=torch.float32, device=DEV)
        g = torch.Generator(DEV).manual_seed(1003)
        self.dY_dev = torch.randn(T, m.hidden, dtype=torch.float32, device=DEV, generator=g) / (T * m.hidden)
        self.dX_dev = torch.empty(T, m.hidden, dtype=torch.float32, device=DEV)
        self.dA = {p: torch.zeros(a.shape, dtype=torch.float32, device=DEV) for p, (a, b) in self.lora_np.items()}
        self.dB = {p: torch.zeros(b.shape, dtype=torch.float32, device=DEV) for p, (a, b) in self.lora_np.items()}
        self.max_kv = int(kv_len.max()) + 1
        self._ft_done = []

    # ---- the two tasks
    def decode_launch(self, stream, batch=None, kv_len_dev=None, max_kv=None):
        """One decode step of the workload's batch (or of `batch` sequences at the given cached lengths)."""
        self.ctx.decode_step(batch=batch or self.B, kv_len=self.kv_len_dev if kv_len_dev is None else kv_len_dev,
                             page_table=self.table_dev, max_pages=self.max_pages, max_kv_len=max_kv or self.max_kv,
                             x_in=self.x_dev, x_out=self.y_dev, stream=stream)

    def finetune_unit(self, stream):
        """Forward + backward of one micro-batch; keeps at most in_flight - 2 units pending (their pool memory is
        released by events)."""
        lim = self.in_flight - 2
        if len(self._ft_done) >= lim:
            self._ft_done[-lim].synchronize()
        sv = self.ctx.lora_fwd(0, self.X_dev, self.Y_dev, self.ft.micro_batch, self.ft.seq_len, stream=stream)
        self.ctx.lora_bwd(0, self.dY_dev, self.dX_dev, sv, self.dA, self.dB, stream=stream)
        ev = torch.cuda.Event()
        ev.record(stream)
        self._ft_done.append(ev)
        if len(self._ft_done) > 64:
            del self._ft_done[:32]

    def drain(self):
        """Waits for the finetune units issued so far and lets go of their events (call before destroying a stream
        they ran on: an event must not be asked about after its stream is gone)."""
        for ev in self._ft_done:
            ev.synchronize()
        self._ft_done = []

    def decode_bytes(self, batch=None, kv_len=None):
        kv = self.kv_len if kv_len is None else kv_len
        return 2 * self.m.layer_params + int(sum(int(n) + 1 for n in kv[: batch or self.B])) * 2 * self.m.kv_row_bytes
