"""ctypes binding of libharli.so: same names as include/harli.h, argument marshalling only.

Every step of the path runs inside the HIP library; this module converts Python
values to C structs and raises on a non-zero status.  It fails loudly if the
library has not been built (`python -m paper_2511_11729_amd.build`).
"""
from __future__ import annotations

import ctypes as C
import sys
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libharli.so")

HARLI_OK, HARLI_ERR_INVALID, HARLI_ERR_OOM, HARLI_ERR_STATE, HARLI_ERR_HIP = range(5)
HARLI_BF16, HARLI_F32 = 0, 1
CLS_KV_PAGE, CLS_TENSOR, CLS_SMALL, CLS_AUTO = range(4)
TARGET_BITS = {"q": 1, "k": 2, "v": 4, "o": 8, "gate": 16, "up": 32, "down": 64}
TARGET_ORDER = ("q", "k", "v", "o", "gate", "up", "down")


class HarliError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("harli status %d: %s" % (status, msg))
        self.status = status


class PoolCfg(C.Structure):
    _fields_ = [("block_bytes", C.c_size_t), ("n_layers", C.c_int32), ("page_tokens", C.c_int32),
                ("kv_row_bytes", C.c_size_t), ("small_pool_bytes", C.c_size_t), ("small_granule", C.c_size_t),
                ("kv_reserve_chunks", C.c_int32)]


class Alloc(C.Structure):
    _fields_ = [("cls", C.c_int32), ("page", C.c_int32), ("offset", C.c_size_t), ("bytes", C.c_size_t),
                ("ptr", C.c_void_p)]


class PoolStats(C.Structure):
    _fields_ = [("n_chunks", C.c_int32), ("free_chunks", C.c_int32), ("kv_chunks", C.c_int32),
                ("tensor_chunks", C.c_int32), ("pages_per_block", C.c_int32), ("blocks_per_chunk", C.c_int32),
                ("kv_pages_live", C.c_int64), ("tensor_blocks_live", C.c_int64), ("small_bytes_live", C.c_size_t),
                ("requested_bytes_live", C.c_size_t), ("reserved_bytes_live", C.c_size_t),
                ("small_fallbacks", C.c_int64), ("pending_frees", C.c_int64)]


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int32), ("max_batch", C.c_int32), ("max_seq_len", C.c_int32),
                ("max_ft_tokens", C.c_int32), ("memory_in_pool", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2", "bq", "bk", "bv")]


class Weights(C.Structure):
    _fields_ = [("layers", C.POINTER(LayerWeights)), ("emb", C.c_void_p), ("g_final", C.c_void_p), ("w_lm", C.c_void_p)]


class LoraCfg(C.Structure):
    _fields_ = [("rank", C.c_int32), ("alpha", C.c_float), ("targets", C.c_uint32), ("workspace_in_pool", C.c_int32),
                ("grad_headroom_log2", C.c_int32)]


class DeviceBytes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("decode_weights", "decode_workspace", "finetune_weights", "finetune_workspace",
                                           "head_weights", "head_workspace", "in_pool", "outside_pool")]


class AdamWCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
                ("grad_scale", C.c_float), ("step", C.c_int32), ("zero_grad", C.c_int32)]


class DecodeBatch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("token_ids", C.c_void_p), ("x_in", C.c_void_p), ("x_out", C.c_void_p),
                ("logits", C.c_void_p), ("next_token", C.c_void_p), ("kv_len", C.c_void_p), ("page_table", C.c_void_p),
                ("max_pages", C.c_int32), ("max_kv_len", C.c_int32)]


_lib = None

_SIGS = {
    "harli_status_str": (C.c_char_p, [C.c_int]),
    "harli_last_error": (C.c_char_p, []),
    "harli_version": (C.c_char_p, []),
    "harli_pool_create": (C.c_int, [C.c_void_p, C.c_size_t, C.POINTER(PoolCfg), C.POINTER(C.c_void_p)]),
    "harli_pool_destroy": (None, [C.c_void_p]),
    "harli_pool_alloc": (C.c_int, [C.c_void_p, C.c_int, C.c_size_t, C.POINTER(Alloc)]),
    "harli_pool_alloc_pages": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "harli_pool_free": (C.c_int, [C.c_void_p, C.POINTER(Alloc), C.c_void_p]),
    "harli_pool_free_pages": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p]),
    "harli_pool_kv_addr": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]),
    "harli_pool_stats": (C.c_int, [C.c_void_p, C.POINTER(PoolStats)]),
    "harli_ctx_create": (C.c_int, [C.POINTER(ModelCfg), C.POINTER(Weights), C.c_void_p, C.POINTER(C.c_void_p)]),
    "harli_ctx_destroy": (None, [C.c_void_p]),
    "harli_ctx_check": (C.c_int, [C.c_void_p, C.c_void_p]),
    "harli_lora_attach": (C.c_int, [C.c_void_p, C.POINTER(LoraCfg), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "harli_ctx_device_bytes": (C.c_int, [C.c_void_p, C.c_void_p]),
    "harli_decode_step": (C.c_int, [C.c_void_p, C.POINTER(DecodeBatch), C.c_void_p]),
    "harli_decode_step_static": (C.c_int, [C.c_void_p, C.POINTER(DecodeBatch), C.c_void_p]),
    "harli_decode_step_static_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int32]),
    "harli_lora_fwd": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                 C.POINTER(C.c_void_p), C.c_void_p]),
    "harli_lora_bwd": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]),
    "harli_saved_release": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "harli_saved_bytes": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]),
    "harli_prof_enable": (C.c_int, [C.c_int32]),
    "harli_prof_collect": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "harli_head_fwd_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "harli_adamw_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(AdamWCfg),
                                   C.c_void_p]),
    "harli_pool_reserve_chunks_for": (C.c_int, [C.c_void_p, C.c_double, C.c_double, C.c_int32, C.POINTER(C.c_int32)]),
    "harli_pool_set_reserve": (C.c_int, [C.c_void_p, C.c_int32]),
    "harli_pool_pressure": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32)]),
    "harli_pred_create": (C.c_int, [C.c_int32, C.POINTER(C.c_void_p)]),
    "harli_pred_destroy": (None, [C.c_void_p]),
    "harli_pred_add_solo": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_double]),
    "harli_pred_add_colo": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double]),
    "harli_pred_set_scale": (C.c_int, [C.c_void_p, C.c_int32, C.c_double]),
    "harli_pred_get_scale": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]),
    "harli_pred_observe": (C.c_int, [C.c_void_p, C.c_int32, C.c_double, C.c_double, C.c_double]),
    "harli_pred_fit": (C.c_int, [C.c_void_p]),
    "harli_pred_solo_coef": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]),
    "harli_pred_solo_coef_upper": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]),
    "harli_pred_set_batch_split": (C.c_int, [C.c_void_p, C.c_int32]),
    "harli_decode_tiled_min_batch": (C.c_int32, []),
    "harli_pred_colo_coef": (C.c_int, [C.c_void_p, C.POINTER(C.c_double)]),
    "harli_pred_set_colo_floor": (C.c_int, [C.c_void_p, C.c_int32]),
    "harli_pred_solo": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]),
    "harli_pred_colo": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]),
    "harli_sched_create": (C.c_int, [C.c_void_p, C.c_double, C.c_int32, C.POINTER(C.c_void_p)]),
    "harli_sched_destroy": (None, [C.c_void_p]),
    "harli_sched_step": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "harli_sched_pick": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                   C.POINTER(C.c_double)]),
    "harli_cu_stream_create": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]),
    "harli_cu_stream_destroy": (C.c_int, [C.c_void_p]),
    "harli_dbg_read_bandwidth": (C.c_int, [C.c_void_p, C.c_size_t, C.c_int32, C.POINTER(C.c_double), C.c_void_p]),
    "harli_ft_window_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "harli_ft_window_resize": (C.c_int, [C.c_void_p, C.c_int32]),
    "harli_ft_window_disable": (C.c_int, [C.c_void_p]),
    "harli_ft_window_ready": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "harli_ft_window_stats": (C.c_int, [C.c_void_p, C.c_void_p]),
    "harli_ft_window_advise": (C.c_int, [C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                          C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "harli_dbg_window_plan": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "harli_dbg_gemm2": (C.c_int, [C.c_void_p, C.c_void_p]),
    "harli_dbg_gemm2_plan": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "harli_dbg_decode_large_min_batch": (None, [C.c_int32]),
    "harli_dbg_decode_gemm_plan": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.POINTER(C.c_int64)]),
    "harli_dbg_decode_gemm_time": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.c_void_p]),
}


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libharli.so is missing: run `python -m paper_2511_11729_amd.build` "
                               "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(status: int) -> None:
    if status != HARLI_OK:
        raise HarliError(status, lib().harli_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


# ----------------------------------------------------------------------------- pool
class Pool:
    """harli_pool_* over a caller-owned slab (a torch uint8 tensor or a raw address)."""

    def __init__(self, slab, slab_bytes: int, *, block_bytes: int = 2 << 20, n_layers: int, page_tokens: int = 16,
                 kv_row_bytes: int, small_pool_bytes: int = 0, small_granule: int = 2048, kv_reserve_chunks: int = 0):
        self._slab = slab
        self.cfg = PoolCfg(block_bytes, n_layers, page_tokens, kv_row_bytes, small_pool_bytes, small_granule,
                           kv_reserve_chunks)
        self.handle = C.c_void_p()
        _check(lib().harli_pool_create(_ptr(slab), slab_bytes, C.byref(self.cfg), C.byref(self.handle)))

    def close(self):
        if self.handle:
            # contexts built on the pool hold it too (the library counts them): the garbage collector may finalise a
            # pool before its contexts
            lib().harli_pool_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            if sys.is_finalizing():   # the HIP runtime may already be gone: let the process exit reclaim everything
                return
            self.close()
        except Exception:
            pass

    def alloc(self, cls: int, n: int = 0) -> Alloc:
        a = Alloc()
        _check(lib().harli_pool_alloc(self.handle, cls, n, C.byref(a)))
        return a

    def alloc_pages(self, n: int) -> List[int]:
        ids = (C.c_int32 * max(n, 1))()
        _check(lib().harli_pool_alloc_pages(self.handle, n, ids))
        return list(ids[:n])

    def free(self, a: Alloc, event=None) -> None:
        _check(lib().harli_pool_free(self.handle, C.byref(a), _event(event)))

    def free_pages(self, ids: Sequence[int], event=None) -> None:
        arr = (C.c_int32 * max(len(ids), 1))(*ids)
        _check(lib().harli_pool_free_pages(self.handle, len(ids), arr, _event(event)))

    def kv_addr(self, page: int, layer: int, kv: int) -> int:
        off = C.c_size_t()
        _check(lib().harli_pool_kv_addr(self.handle, page, layer, kv, C.byref(off)))
        return off.value

    def stats(self) -> PoolStats:
        s = PoolStats()
        _check(lib().harli_pool_stats(self.handle, C.byref(s)))
        return s

    def reserve_chunks_for(self, release_time: float, slo: float, max_bs: int) -> int:
        """Chunks holding Memory_reserved = (T / SLO) * max_bs * Mem_kv (Sec. 4.4)."""
        n = C.c_int32()
        _check(lib().harli_pool_reserve_chunks_for(self.handle, release_time, slo, max_bs, C.byref(n)))
        return n.value

    def set_reserve(self, chunks: int) -> None:
        _check(lib().harli_pool_set_reserve(self.handle, chunks))

    def pressure(self) -> int:
        """Chunks the finetune task should relinquish now."""
        n = C.c_int32()
        _check(lib().harli_pool_pressure(self.handle, C.byref(n)))
        return n.value


def _event(e) -> Optional[int]:
    if e is None:
        return None
    if isinstance(e, int):
        return e
    return e.cuda_event


# ----------------------------------------------------------------------------- context
class Context:
    """harli_ctx_* ; `layers` is a list of dicts of torch tensors (wq..wd, g1, g2)."""

    def __init__(self, pool: Pool, *, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab=0,
                 rms_eps=1e-6, rope_base=10000.0, dtype=HARLI_BF16, max_batch=16, max_seq_len=4096,
                 max_ft_tokens=0, layers, emb=None, g_final=None, w_lm=None, memory_in_pool=False):
        self.pool = pool
        self._keep = (layers, emb, g_final, w_lm)
        self.cfg = ModelCfg(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, rms_eps, rope_base, dtype,
                            max_batch, max_seq_len, max_ft_tokens, int(bool(memory_in_pool)))
        arr = (LayerWeights * n_layers)()
        for i, lw in enumerate(layers):
            for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2"):
                setattr(arr[i], n, _ptr(lw[n]))
            for n in ("bq", "bk", "bv"):                      # optional frozen biases (fp32)
                setattr(arr[i], n, _ptr(lw.get(n)))
        w = Weights(arr, _ptr(emb), _ptr(g_final), _ptr(w_lm))
        self.handle = C.c_void_p()
        _check(lib().harli_ctx_create(C.byref(self.cfg), C.byref(w), pool.handle, C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib().harli_ctx_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            if sys.is_finalizing():   # the HIP runtime may already be gone: let the process exit reclaim everything
                return
            self.close()
        except Exception:
            pass

    def check(self, stream=None) -> None:
        _check(lib().harli_ctx_check(self.handle, _stream(stream)))

    # ---- window over the finetune task's frozen weights (harli_ft_window_*)
    def ft_window_enable(self, n_slots: int) -> None:
        _check(lib().harli_ft_window_enable(self.handle, n_slots))

    def ft_window_resize(self, n_slots: int) -> None:
        _check(lib().harli_ft_window_resize(self.handle, n_slots))

    def ft_window_disable(self) -> None:
        _check(lib().harli_ft_window_disable(self.handle))

    def ft_window_ready(self, layer: int, backward: bool) -> bool:
        r = C.c_int32(0)
        _check(lib().harli_ft_window_ready(self.handle, layer, int(bool(backward)), C.byref(r)))
        return bool(r.value)

    def ft_window_stats(self) -> "WindowStats":
        st = WindowStats()
        _check(lib().harli_ft_window_stats(self.handle, C.byref(st)))
        return st

    def device_bytes(self) -> "DeviceBytes":
        b = DeviceBytes()
        _check(lib().harli_ctx_device_bytes(self.handle, C.byref(b)))
        return b

    def lora_attach(self, rank: int, alpha: float, targets: Sequence[str], A, B, workspace_in_pool: bool = False,
                    grad_headroom_log2: int = 0) -> None:
        """A, B: per layer a dict target -> torch tensor."""
        n_layers = self.cfg.n_layers
        self._lora_keep = (A, B)
        pa = (C.c_void_p * (n_layers * 7))()
        pb = (C.c_void_p * (n_layers * 7))()
        mask = 0
        for t in targets:
            mask |= TARGET_BITS[t]
        for l in range(n_layers):
            for i, t in enumerate(TARGET_ORDER):
                if t in targets:
                    pa[l * 7 + i] = _ptr(A[l][t])
                    pb[l * 7 + i] = _ptr(B[l][t])
        cfg = LoraCfg(rank, alpha, mask, int(bool(workspace_in_pool)), grad_headroom_log2)
        _check(lib().harli_lora_attach(self.handle, C.byref(cfg), pa, pb))

    def decode_step(self, *, batch, kv_len, page_table, max_pages, max_kv_len, token_ids=None, x_in=None, x_out=None,
                    logits=None, next_token=None, stream=None) -> None:
        b = DecodeBatch(batch, _ptr(token_ids), _ptr(x_in), _ptr(x_out), _ptr(logits), _ptr(next_token), _ptr(kv_len),
                        _ptr(page_table), max_pages, max_kv_len)
        _check(lib().harli_decode_step(self.handle, C.byref(b), _stream(stream)))

    def decode_step_static(self, *, batch, kv_len, page_table, max_pages, max_kv_len, token_ids=None, x_in=None, x_out=None,
                           logits=None, next_token=None, stream=None) -> None:
        """harli_decode_step on the library's static scratch array: the call allocates nothing."""
        b = DecodeBatch(batch, _ptr(token_ids), _ptr(x_in), _ptr(x_out), _ptr(logits), _ptr(next_token), _ptr(kv_len),
                        _ptr(page_table), max_pages, max_kv_len)
        _check(lib().harli_decode_step_static(self.handle, C.byref(b), _stream(stream)))

    def decode_step_static_bytes(self, batch: int, max_kv_len: int) -> int:
        return int(lib().harli_decode_step_static_bytes(self.handle, batch, max_kv_len))

    def lora_fwd(self, layer: int, X, Y, B_f: int, S: int, stream=None) -> int:
        saved = C.c_void_p()
        _check(lib().harli_lora_fwd(self.handle, layer, _ptr(X), _ptr(Y), B_f, S, C.byref(saved), _stream(stream)))
        return saved.value

    def lora_bwd(self, layer: int, dY, dX, saved: int, dA, dB, stream=None) -> None:
        """dA, dB: dict target -> fp32 torch tensor (accumulated into)."""
        pa = (C.c_void_p * 7)()
        pb = (C.c_void_p * 7)()
        for i, t in enumerate(TARGET_ORDER):
            if t in dA:
                pa[i] = _ptr(dA[t])
                pb[i] = _ptr(dB[t])
        _check(lib().harli_lora_bwd(self.handle, layer, _ptr(dY), _ptr(dX), saved, pa, pb, _stream(stream)))

    def head_fwd_bwd(self, x, targets, loss, dx, stream=None) -> None:
        """Output layer + next-token cross entropy: x fp32 [T, hidden], targets int32 [T] (-1 = not counted), loss fp32
        scalar tensor, dx fp32 [T, hidden]."""
        _check(lib().harli_head_fwd_bwd(self.handle, _ptr(x), _ptr(targets), x.shape[0], _ptr(loss), _ptr(dx), _stream(stream)))

    def saved_release(self, saved: int, stream=None) -> None:
        _check(lib().harli_saved_release(self.handle, saved, _stream(stream)))

    def saved_bytes(self, B_f: int, S: int) -> int:
        n = C.c_size_t()
        _check(lib().harli_saved_bytes(self.handle, B_f, S, C.byref(n)))
        return n.value


def adamw_step(master, m, v, grad, param_bf16, *, step: int, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
               grad_scale=1.0, zero_grad=False, stream=None) -> None:
    """AdamW on device tensors: fp32 master / moments / gradient, optional bf16 copy rewritten from the master."""
    cfg = AdamWCfg(lr, beta1, beta2, eps, weight_decay, grad_scale, step, int(zero_grad))
    _check(lib().harli_adamw_step(_ptr(master), _ptr(m), _ptr(v), _ptr(grad), _ptr(param_bf16), master.numel(), C.byref(cfg),
                                  _stream(stream)))


# ----------------------------------------------------------------------------- predictor / scheduler (harli_sched.h)
class Predictor:
    """harli_pred_* / harli_sched_pick: Eq. 1 per compute-unit level, Eq. 2 overall, closest-below-target choice."""

    def __init__(self, n_levels: int = 10):
        self.n_levels = n_levels
        self.handle = C.c_void_p()
        _check(lib().harli_pred_create(n_levels, C.byref(self.handle)))

    def close(self):
        if self.handle:
            lib().harli_pred_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            if sys.is_finalizing():   # the HIP runtime may already be gone: let the process exit reclaim everything
                return
            self.close()
        except Exception:
            pass

    def add_solo(self, level: int, bs: int, seqlen: int, latency: float) -> None:
        _check(lib().harli_pred_add_solo(self.handle, level, bs, seqlen, latency))

    def add_colo(self, infer_level: int, ft_level: int, latency_colo: float, latency_solo: float) -> None:
        _check(lib().harli_pred_add_colo(self.handle, infer_level, ft_level, latency_colo, latency_solo))

    def fit(self) -> None:
        _check(lib().harli_pred_fit(self.handle))

    def set_scale(self, level: int, scale: float) -> None:
        """Calibration factor on every prediction at `level` (1 by default)."""
        _check(lib().harli_pred_set_scale(self.handle, level, C.c_double(scale)))

    def get_scale(self, level: int) -> float:
        v = C.c_double(0.0)
        _check(lib().harli_pred_get_scale(self.handle, level, C.byref(v)))
        return v.value

    def observe(self, level: int, predicted_ms: float, measured_ms: float, weight: float) -> None:
        """Folds one measured decode step into the calibration factor of `level` (predicted_ms: without the factor)."""
        _check(lib().harli_pred_observe(self.handle, level, C.c_double(predicted_ms), C.c_double(measured_ms),
                                        C.c_double(weight)))

    def solo_coef(self, level: int):
        c = (C.c_double * 3)()
        _check(lib().harli_pred_solo_coef(self.handle, level, c))
        return tuple(c)

    def solo_coef_upper(self, level: int):
        """Eq. 1 coefficients of `level` for batches from the split on (those of solo_coef without a split)."""
        c = (C.c_double * 3)()
        _check(lib().harli_pred_solo_coef_upper(self.handle, level, c))
        return tuple(c)

    def set_batch_split(self, bs_split: int) -> None:
        """Batches from bs_split on get Eq. 1 coefficients of their own (0: one line per level, as printed)."""
        _check(lib().harli_pred_set_batch_split(self.handle, bs_split))

    def set_colo_floor(self, enabled: bool) -> None:
        _check(lib().harli_pred_set_colo_floor(self.handle, 1 if enabled else 0))

    def colo_coef(self):
        c = (C.c_double * 2)()
        _check(lib().harli_pred_colo_coef(self.handle, c))
        return tuple(c)

    def solo(self, level: int, bs: int, seqlen: int) -> float:
        v = C.c_double()
        _check(lib().harli_pred_solo(self.handle, level, bs, seqlen, C.byref(v)))
        return v.value

    def colo(self, infer_level: int, ft_level: int, bs: int, seqlen: int) -> float:
        v = C.c_double()
        _check(lib().harli_pred_colo(self.handle, infer_level, ft_level, bs, seqlen, C.byref(v)))
        return v.value

    def pick(self, bs: int, seqlen: int, slo: float):
        """(infer_level, ft_level, predicted latency); ft_level 0 = finetune paused, inference on every compute unit."""
        i, f, v = C.c_int32(), C.c_int32(), C.c_double()
        _check(lib().harli_sched_pick(self.handle, bs, seqlen, slo, C.byref(i), C.byref(f), C.byref(v)))
        return i.value, f.value, v.value


SCHED_KEEP, SCHED_REPLAN, SCHED_PAUSED, SCHED_STARVED = 0, 1, 2, 3


class SchedDecision(C.Structure):
    _fields_ = [("infer_level", C.c_int32), ("ft_level", C.c_int32), ("action", C.c_int32), ("predicted", C.c_double)]


class Scheduler:
    """harli_sched_create / step: one allocation decision per decode phase.  Keeps the predictor alive."""

    def __init__(self, pred: Predictor, slo: float, refresh_phases: int = 0):
        self.pred = pred
        h = C.c_void_p()
        _check(lib().harli_sched_create(pred.handle, slo, refresh_phases, C.byref(h)))
        self.handle = h

    def close(self):
        if self.handle:
            lib().harli_sched_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            if sys.is_finalizing():   # the HIP runtime may already be gone: let the process exit reclaim everything
                return
            self.close()
        except Exception:
            pass

    def step(self, bs: int, seqlen: int, ft_ready: bool = True):
        """(infer_level, ft_level, predicted latency, action)."""
        d = SchedDecision()
        _check(lib().harli_sched_step(self.handle, bs, seqlen, int(bool(ft_ready)), C.byref(d)))
        return d.infer_level, d.ft_level, d.predicted, d.action


def cu_stream_create(cu_first: int, cu_count: int) -> int:
    """hipStream_t (as an integer) restricted to compute units [cu_first, cu_first + cu_count)."""
    h = C.c_void_p()
    _check(lib().harli_cu_stream_create(cu_first, cu_count, C.byref(h)))
    return h.value


def cu_stream_destroy(stream: int) -> None:
    _check(lib().harli_cu_stream_destroy(stream))


class DbgGemm2Desc(C.Structure):
    _fields_ = [("M", C.c_int32), ("nseg", C.c_int32), ("nout", C.c_int32), ("tiles_n", C.c_int32), ("half", C.c_int32),
                ("epi", C.c_int32), ("tile_rows", C.c_int32), ("reps", C.c_int32), ("alpha", C.c_float),
                ("A", C.c_void_p * 12), ("lda", C.c_int64 * 12), ("K", C.c_int32 * 12), ("B", C.c_void_p * 12),
                ("b_rows", C.c_int32 * 12), ("B2", C.c_void_p * 12), ("b2_rows", C.c_int32 * 12), ("tile0", C.c_int32 * 12),
                ("tile1", C.c_int32 * 12), ("pair", C.c_int32 * 12), ("out_tile0", C.c_int32 * 3), ("out_n", C.c_int32 * 3),
                ("cb", C.c_void_p * 3), ("ldcb", C.c_int64 * 3), ("cf", C.c_void_p * 3), ("res", C.c_void_p * 3),
                ("ldcf", C.c_int64 * 3), ("e0", C.c_void_p), ("e1", C.c_void_p), ("o0", C.c_void_p), ("o1", C.c_void_p),
                ("lde", C.c_int64), ("overflow_flag", C.c_void_p), ("tflops", C.POINTER(C.c_double)),
                ("shader_mhz", C.POINTER(C.c_double)), ("n_cu", C.c_int32)]


def decode_tiled_min_batch() -> int:
    """Smallest batch whose decode steps run the tiled GEMMs."""
    return int(lib().harli_decode_tiled_min_batch())


def dbg_decode_large_min_batch(batch: int) -> None:
    """Measurement hook: the smallest batch whose decode steps run the tiled GEMMs (0: the library's own)."""
    lib().harli_dbg_decode_large_min_batch(batch)


def dbg_decode_gemm_plan(batch: int, n_rows: int, n_mat: int, K: int, n_cu: int, ws_bytes: int) -> dict:
    """How one GEMM of a decode step above 32 sequences is cut (host logic only)."""
    out = (C.c_int64 * 7)()
    _check(lib().harli_dbg_decode_gemm_plan(batch, n_rows, n_mat, K, n_cu, ws_bytes, out))
    return dict(zip(("FM", "tiles_m", "Mpad", "tiles_n", "ksplit", "rounds", "part_bytes"), [int(v) for v in out]))


def dbg_decode_gemm_time(batch: int, n_rows: int, n_mat: int, K: int, ksplit: int = 0, reps: int = 10, stream=None) -> dict:
    """Average microseconds of the two launches of one large-batch decode GEMM on operands the call allocates."""
    out = (C.c_float * 4)()
    _check(lib().harli_dbg_decode_gemm_time(batch, n_rows, n_mat, K, ksplit, reps, out, _stream(stream)))
    return {"gemm_us": float(out[0]), "epilogue_us": float(out[1]), "ksplit": int(out[2]), "FM": int(out[3])}


def dbg_gemm2_plan(M: int, tiles_n: int, tile_rows: int, n_cu: int) -> dict:
    """The launch grid of the weight GEMM (host logic): GM, GN, total, chunk, grid, rounds."""
    out = (C.c_int32 * 6)()
    _check(lib().harli_dbg_gemm2_plan(M, tiles_n, tile_rows, n_cu, out))
    return dict(zip(("GM", "GN", "total", "chunk", "grid", "rounds"), list(out)))


def dbg_gemm2(M, segs, outs, *, half=True, epi=0, alpha=1.0, tile_rows=0, reps=0, e0=None, e1=None, o0=None, o1=None, lde=0,
              overflow_flag=None, stream=None, n_cu=0):
    """Test hook for the finetune unit's weight GEMM.  segs: dicts with A (device [M, K], 16-bit), optional lda,
    B (device [rows, K] row-major weight side; the hook blocks it), optional B2 and pair, optional tile0 / tile1.
    outs: dicts with N, tile0 and cb (16-bit) or cf (+ res), optional ld.  Tiles are 256 columns (128 + 128 for
    pairs).  Returns (TFLOP/s, shader MHz) when reps > 1."""
    d = DbgGemm2Desc()
    d.M, d.nseg, d.nout, d.half, d.epi, d.tile_rows, d.reps, d.alpha = M, len(segs), len(outs), int(half), epi, tile_rows, reps, alpha
    width = 128 if epi == 3 else 256
    tiles = 0
    for o, q in enumerate(outs):
        d.out_tile0[o] = q.get("tile0", tiles)
        d.out_n[o] = q["N"]
        tiles = d.out_tile0[o] + -(-q["N"] // width)
        if q.get("cb") is not None:
            d.cb[o], d.ldcb[o] = _ptr(q["cb"]), q.get("ld", q["cb"].shape[1])
        if q.get("cf") is not None:
            d.cf[o], d.ldcf[o] = _ptr(q["cf"]), q.get("ld", q["cf"].shape[1])
        if q.get("res") is not None:
            d.res[o] = _ptr(q["res"])
    d.tiles_n = tiles
    for s, q in enumerate(segs):
        A = q["A"]
        d.A[s], d.lda[s], d.K[s] = _ptr(A), q.get("lda", A.shape[1]), q.get("K", A.shape[1])
        if q.get("B") is not None:
            d.B[s], d.b_rows[s] = _ptr(q["B"]), q["B"].shape[0]
        if q.get("B2") is not None:
            d.B2[s], d.b2_rows[s] = _ptr(q["B2"]), q["B2"].shape[0]
        d.pair[s] = int(q.get("pair", 0))
        d.tile0[s], d.tile1[s] = q.get("tile0", 0), q.get("tile1", tiles)
    d.e0, d.e1, d.o0, d.o1, d.lde = _ptr(e0), _ptr(e1), _ptr(o0), _ptr(o1), lde
    d.overflow_flag = _ptr(overflow_flag)
    d.n_cu = n_cu
    t, f = C.c_double(0.0), C.c_double(0.0)
    if reps > 1:
        d.tflops, d.shader_mhz = C.pointer(t), C.pointer(f)
    _check(lib().harli_dbg_gemm2(C.byref(d), _stream(stream)))
    return t.value, f.value


class WindowStats(C.Structure):
    _fields_ = [("slots", C.c_int32), ("slot_bytes", C.c_size_t), ("host_bytes", C.c_size_t), ("h2d_bytes", C.c_int64),
                ("hits", C.c_int64), ("misses", C.c_int64), ("refills", C.c_int64)]


def ft_window_advise(slots: int, max_slots: int, slot_chunks: int, free_chunks: int, need_chunks: int, pressed: bool,
                     calm: int):
    """(target slots, updated calm count) of harli_ft_window_advise."""
    c, t = C.c_int32(calm), C.c_int32(0)
    _check(lib().harli_ft_window_advise(slots, max_slots, slot_chunks, free_chunks, need_chunks, int(bool(pressed)),
                                        C.byref(c), C.byref(t)))
    return t.value, c.value


def dbg_window_plan(n_layers: int, n_slots: int, items):
    """(slot, miss, refill) lists of the library's window residency plan driven through `items`."""
    n = len(items)
    arr = (C.c_int32 * max(n, 1))(*items)
    slot, miss, refill = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
    _check(lib().harli_dbg_window_plan(n_layers, n_slots, arr, n, slot, miss, refill))
    return list(slot[:n]), list(miss[:n]), list(refill[:n])


def dbg_read_bandwidth(buf, mode: int, stream=None) -> float:
    """Measured read rate in GB/s over the uint8 device tensor `buf`: mode 0 streams it (HBM), mode 1 re-reads
    shared regions the way GEMM workgroups do (L2)."""
    g = C.c_double()
    _check(lib().harli_dbg_read_bandwidth(_ptr(buf), buf.numel() * buf.element_size(), mode, C.byref(g), _stream(stream)))
    return g.value


def prof_enable(every: int) -> None:
    """Time every `every`-th launch of the finetune GEMM from now on (1 or True: all; 0 or False: off)."""
    _check(lib().harli_prof_enable(int(every)))


def prof_collect():
    """(gemm flops, gemm milliseconds, launches) since the last call; waits for the recorded events."""
    f, t, n = C.c_double(), C.c_double(), C.c_int64()
    _check(lib().harli_prof_collect(C.byref(f), C.byref(t), C.byref(n)))
    return f.value, t.value, n.value
