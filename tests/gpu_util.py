"""Helpers for the GPU parity tests: move seeded inputs to the device, lay out the paged
KV cache through the pool, and run the oracle on the same bytes."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from oracle import harli_oracle as O
from paper_2511_11729_amd import binding as hb

DEV = "cuda:0"
PROJ = dict(q="wq", k="wk", v="wv", o="wo", gate="wg", up="wu", down="wd")


def to_dev(a: np.ndarray, dtype: str):
    """Storage-typed device tensor of a float32 array (bf16 values are already representable)."""
    if dtype == "bf16":
        bits = wl.bf16_bits(a).view(np.int16).reshape(a.shape)
        return torch.from_numpy(bits).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


def f32_dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


def shapes_of(m: wl.ModelCfg) -> O.Shapes:
    return O.Shapes(m.hidden, m.n_q, m.n_kv, m.head_dim, m.ffn, m.rms_eps, m.rope_base)


def rel_fro(a, ref):
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


def max_abs_ratio(a, ref):
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(a - ref)) / max(np.max(np.abs(ref)), 1e-300))


def assert_close(a, ref, what, max_ratio=2e-2, fro=5e-3):
    """The bf16 bar: max-abs error <= 2e-2 * max|ref| and relative Frobenius error <= 5e-3."""
    assert np.all(np.isfinite(np.asarray(a))), what + ": non-finite output"
    mr, fr = max_abs_ratio(a, ref), rel_fro(a, ref)
    assert mr <= max_ratio and fr <= fro, "%s: max-abs ratio %.3e (<= %.1e), rel-Fro %.3e (<= %.1e)" % (what, mr, max_ratio, fr, fro)
    return mr, fr


class DecodeCase:
    """One decode step on both sides.  `model` may differ from the workload's (shape variants)."""

    def __init__(self, w: wl.Workload, model: wl.ModelCfg, lengths, *, full_model=False, block_bytes=2 << 20,
                 small_pool_bytes=0, extra_chunks=1, max_batch=None, reserve=0, tweak=None,
                 memory_in_pool=False):
        self.w, self.m = w, model
        m = model
        self.B = B = len(lengths)
        self.dtype = m.dtype
        eb = m.elem_bytes
        self.layers_np = [wl.make_layer_weights(w, l, m) for l in range(m.n_layers)]
        self.extras_np = wl.make_model_extras(w, m) if full_model else None
        if tweak is not None:
            tweak(self)          # edit the host-side weights before the context reads them
        self.x_np, self.kv_len, self.kv_np = wl.make_decode_inputs(w, B, m, lengths)
        P = 16
        n_pages = [(int(n) + 1 + P - 1) // P for n in self.kv_len]
        self.max_pages = max(n_pages) + 1
        total_pages = sum(n_pages)
        page_bytes = P * m.kv_row_bytes
        ppb = block_bytes // page_bytes
        chunk_bytes = m.n_layers * 2 * block_bytes
        n_chunks = -(-total_pages // ppb) + extra_chunks
        self.slab_bytes = small_pool_bytes + n_chunks * chunk_bytes
        self.geom = O.PoolGeometry(block_bytes, m.n_layers, P, m.kv_row_bytes, small_pool_bytes, self.slab_bytes)
        self.slab = torch.zeros(self.slab_bytes, dtype=torch.uint8, device=DEV)
        self.pool = hb.Pool(self.slab, self.slab_bytes, block_bytes=block_bytes, n_layers=m.n_layers, page_tokens=P,
                            kv_row_bytes=m.kv_row_bytes, small_pool_bytes=small_pool_bytes, kv_reserve_chunks=reserve)
        ids = np.array(self.pool.alloc_pages(total_pages), np.int64)
        self.page_ids = ids
        ids = ids[wl.page_order(w, total_pages)]             # scatter logical pages over physical ones
        self.table = np.full((B, self.max_pages), -1, np.int32)
        k = 0
        for b in range(B):
            self.table[b, : n_pages[b]] = ids[k: k + n_pages[b]]
            k += n_pages[b]
        # slab image (host), written with the oracle's address function
        np_elem = np.uint16 if m.dtype == "bf16" else np.float32
        img = np.zeros(self.slab_bytes // eb, np_elem)
        d = m.head_dim
        for l in range(m.n_layers):
            for b in range(B):
                K, V = self.kv_np[l][b]
                n = K.shape[0]
                for which, T in ((0, K), (1, V)):
                    enc = wl.bf16_bits(T).reshape(T.shape) if m.dtype == "bf16" else T
                    for lp in range((n + P - 1) // P):
                        t0, t1 = lp * P, min(n, lp * P + P)
                        for c in range(m.n_kv):
                            off = self.geom.head_offset(int(self.table[b, lp]), l, which, c, 0, d * eb) // eb
                            img[off: off + (t1 - t0) * d] = enc[t0:t1, c, :].reshape(-1)
        self.img0 = img
        self.slab.copy_(torch.from_numpy(img.view(np.uint8)))
        # device tensors
        self.layers_dev = []
        for L in self.layers_np:
            dl = {n: to_dev(L[n], m.dtype) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
            dl["g1"], dl["g2"] = f32_dev(L["g1"]), f32_dev(L["g2"])
            for bn in ("bq", "bk", "bv"):
                if bn in L:
                    dl[bn] = f32_dev(L[bn])
            self.layers_dev.append(dl)
        kw = {}
        if full_model:
            self.emb_dev = to_dev(self.extras_np["emb"], m.dtype)
            self.gf_dev = f32_dev(self.extras_np["gf"])
            self.wlm_dev = to_dev(self.extras_np["wlm"], m.dtype)
            kw = dict(emb=self.emb_dev, g_final=self.gf_dev, w_lm=self.wlm_dev, vocab=m.vocab)
        self.ctx = hb.Context(self.pool, n_layers=m.n_layers, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv,
                              head_dim=m.head_dim, ffn=m.ffn, rms_eps=m.rms_eps, rope_base=m.rope_base,
                              dtype=hb.HARLI_BF16 if m.dtype == "bf16" else hb.HARLI_F32,
                              max_batch=max_batch or B, max_seq_len=int(max(self.kv_len)) + 8,
                              layers=self.layers_dev, memory_in_pool=memory_in_pool, **kw)
        self.kv_len_dev = torch.from_numpy(self.kv_len.astype(np.int32)).to(DEV)
        self.table_dev = torch.from_numpy(self.table).to(DEV)
        self.x_dev = f32_dev(self.x_np)

    # -- GPU ---------------------------------------------------------------------------------
    def run_gpu(self, token_ids=None, stream=None):
        m, B = self.m, self.B
        self.y_dev = torch.empty(B, m.hidden, dtype=torch.float32, device=DEV)
        kw = {}
        if token_ids is not None:
            self.tok_dev = torch.from_numpy(np.asarray(token_ids, np.int32)).to(DEV)
            self.logits_dev = torch.empty(B, m.vocab, dtype=torch.float32, device=DEV)
            self.next_dev = torch.empty(B, dtype=torch.int32, device=DEV)
            kw = dict(token_ids=self.tok_dev, logits=self.logits_dev, next_token=self.next_dev)
        else:
            kw = dict(x_in=self.x_dev)
        self.ctx.decode_step(batch=B, kv_len=self.kv_len_dev, page_table=self.table_dev, max_pages=self.max_pages,
                             max_kv_len=int(max(self.kv_len)) + 1, x_out=self.y_dev, stream=stream, **kw)
        torch.cuda.synchronize()
        self.ctx.check()
        return self.y_dev.cpu().numpy()

    def slab_image(self):
        np_elem = np.uint16 if self.dtype == "bf16" else np.float32
        return self.slab.cpu().numpy().view(np_elem)

    # -- oracle ----------------------------------------------------------------------------------
    def _decode_img(self, img):
        return (wl.bf16_from_bits(img) if self.dtype == "bf16" else img).astype(np.float64)

    def run_oracle(self, token_ids=None):
        m = self.m
        kv = O.PagedKV(self.geom, m.elem_bytes, m.n_kv, m.head_dim, slab=self._decode_img(self.img0))
        self.okv = kv
        sh = shapes_of(m)
        if token_ids is None:
            return O.decode_model_paged(self.x_np, self.layers_np, None, sh, kv, self.kv_len, self.table)
        return O.decode_model_paged(np.asarray(token_ids), self.layers_np, self.extras_np, sh, kv, self.kv_len, self.table)

    def check_cache(self, tol_ratio=2e-2, fro=5e-3):
        """Appended K/V: exactly the oracle's positions changed (bit-exact indexing), values within the bar
        (default: the bf16 one)."""
        img1 = self.slab_image()
        changed_gpu = np.flatnonzero(img1 != self.img0)
        ref = self.okv.slab
        changed_ref = np.flatnonzero(ref != self._decode_img(self.img0))
        assert np.array_equal(changed_gpu, changed_ref), "appended K/V landed at different addresses"
        got = self._decode_img(img1)[changed_ref]
        want = ref[changed_ref]
        assert np.max(np.abs(got - want)) <= tol_ratio * np.max(np.abs(want))
        assert rel_fro(got, want) <= fro
        return len(changed_ref)


class FinetuneCase:
    """One finetune unit (layer forward + backward) on both sides."""

    def __init__(self, w: wl.Workload, model: wl.ModelCfg, lora: wl.LoraCfg, ft: wl.FinetuneCfg, *,
                 block_bytes=2 << 20, small_pool_bytes=8 << 20, zero_b=False, n_chunks=None, sets=1, tweak=None,
                 grad_headroom_log2=0, attach=True, memory_in_pool=False):
        """tweak(case): edits W_np / lora_np / X_np (both sides then see the edited values)."""
        self.w, self.m, self.lora, self.ft = w, model, lora, ft
        m = model
        self.W_np = wl.make_layer_weights(w, 0, m)
        self.lora_np = wl.make_lora(w, 0, m, lora, zero_b=zero_b)
        self.X_np, self.T_np = wl.make_finetune_inputs(w, m, ft)
        if tweak is not None:
            tweak(self)
        T = ft.tokens
        # a first context-free estimate of the pool size: activations + slack
        Z = ft.micro_batch * m.n_q
        est = (T * m.hidden * 12 + T * m.n_q * m.head_dim * 4 + T * m.n_kv * m.head_dim * 4 + T * m.ffn * 6
               + Z * ft.seq_len * ft.seq_len * 2)
        chunk = m.n_layers * 2 * block_bytes
        n_chunks = n_chunks or sets * (est // chunk + 4)   # `sets` micro-batches may be in flight at once
        self.slab_bytes = small_pool_bytes + n_chunks * chunk
        self.slab = torch.zeros(self.slab_bytes, dtype=torch.uint8, device=DEV)
        self.pool = hb.Pool(self.slab, self.slab_bytes, block_bytes=block_bytes, n_layers=m.n_layers,
                            kv_row_bytes=m.kv_row_bytes, small_pool_bytes=small_pool_bytes, kv_reserve_chunks=1)
        self.layer_dev = {n: to_dev(self.W_np[n], m.dtype) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
        self.layer_dev["g1"], self.layer_dev["g2"] = f32_dev(self.W_np["g1"]), f32_dev(self.W_np["g2"])
        for bn in ("bq", "bk", "bv"):
            if bn in self.W_np:
                self.layer_dev[bn] = f32_dev(self.W_np[bn])
        self.ctx = hb.Context(self.pool, n_layers=m.n_layers, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv,
                              head_dim=m.head_dim, ffn=m.ffn, rms_eps=m.rms_eps, rope_base=m.rope_base,
                              dtype=hb.HARLI_BF16 if m.dtype == "bf16" else hb.HARLI_F32, max_batch=1, max_seq_len=16,
                              max_ft_tokens=T, memory_in_pool=memory_in_pool,
                              layers=[self.layer_dev])
        self.A_dev = {p: to_dev(a, m.dtype) for p, (a, b) in self.lora_np.items()}
        self.B_dev = {p: to_dev(b, m.dtype) for p, (a, b) in self.lora_np.items()}
        if attach:
            self.ctx.lora_attach(lora.rank, lora.alpha, lora.targets, [self.A_dev], [self.B_dev],
                                 grad_headroom_log2=grad_headroom_log2)
        self.X_dev = f32_dev(self.X_np.reshape(T, m.hidden))

    def forward_gpu(self, stream=None):
        T, H = self.ft.tokens, self.m.hidden
        self.Y_dev = torch.empty(T, H, dtype=torch.float32, device=DEV)
        self.saved = self.ctx.lora_fwd(0, self.X_dev, self.Y_dev, self.ft.micro_batch, self.ft.seq_len, stream=stream)
        torch.cuda.synchronize()
        return self.Y_dev.cpu().numpy().reshape(self.X_np.shape)

    def backward_gpu(self, dY: np.ndarray, stream=None, accumulate_into=None):
        T, H = self.ft.tokens, self.m.hidden
        self.dY_dev = f32_dev(dY.reshape(T, H))
        self.dX_dev = torch.empty(T, H, dtype=torch.float32, device=DEV)
        if accumulate_into is None:
            self.dA_dev = {p: torch.zeros(a.shape, dtype=torch.float32, device=DEV) for p, (a, b) in self.lora_np.items()}
            self.dB_dev = {p: torch.zeros(b.shape, dtype=torch.float32, device=DEV) for p, (a, b) in self.lora_np.items()}
        self.ctx.lora_bwd(0, self.dY_dev, self.dX_dev, self.saved, self.dA_dev, self.dB_dev, stream=stream)
        torch.cuda.synchronize()
        return (self.dX_dev.cpu().numpy().reshape(self.X_np.shape),
                {p: (self.dA_dev[p].cpu().numpy(), self.dB_dev[p].cpu().numpy()) for p in self.dA_dev})

    def oracle(self):
        sh = shapes_of(self.m)
        Y, saved = O.layer_forward(self.X_np, self.W_np, self.lora_np, self.lora.scale, sh)
        loss, dY = O.mse_loss(Y, self.T_np)
        dX, grads = O.layer_backward(dY, saved, self.W_np, self.lora_np, self.lora.scale, sh)
        return Y, loss, dY, dX, grads
