"""CPU oracle for the decode step and the LoRA finetune layer (TEST INFRASTRUCTURE).

This file is the plain definition of what the HIP library computes, written in
NumPy float64 with no blocking, no online softmax, no fusion and no code shared
with the GPU path.  Only tests, the smoke check and the CPU-baseline leg of the
benchmark may import it; the product never does.

What the paper fixes (Harli, arXiv 2511.11729) is the problem, not the kernels:
  * Sec. 2.1: a decoder-only LLM is an embedding, a stack of transformer layers
    (self-attention + FFN, "mainly matrix multiplications") and an output
    layer; decode produces one token per sequence per step and reuses the KV
    cache written by earlier steps.
  * Sec. 2.1 / 4.1: a PEFT finetune iteration is forward, backward, update;
    LoRA freezes every base parameter and trains only the attached adapters,
    so only adapter gradients (and the gradient w.r.t. the layer input) exist.
  * Sec. 6.1: the finetune model is cut into one sub-model per transformer
    layer whose output (forward) / input gradient (backward) is handed over
    explicitly; `layer_forward` / `layer_backward` are that unit.
  * Sec. 4.1 / 4.2: KV slots are handed out by index from a pre-allocated pool
    laid out as a 2-D grid (row = layer x {K, V}, column = token run); chunk =
    layerNum x 2 blocks.  `PoolGeometry.kv_offset` is that grid.
The layer arithmetic the paper does not spell out (RMSNorm, rotary position
embedding with half-split pairs, SwiGLU, grouped-query attention, LoRA
`y = x W^T + (alpha/r) (x A) B`, MSE / cross-entropy losses) is the textbook
definition; each function below states the formula it implements.

Pins (tests/test_oracle_*.py, CPU only): B = 0 gives the base output; merged
weights W + s (A B)^T give the LoRA output; dX / dA / dB match central finite
differences of the scalar loss; one cached token returns V; equal keys return
mean(V); paged and contiguous caches agree bit for bit for any page
permutation; a decode step equals the last row of the causal forward; RoPE is a
norm-preserving relative rotation; RMSNorm output has unit RMS.  The full
multi-layer model is pinned only as "a stack of the pinned layer" -- parity
with a real checkpoint is unpinned (no weights are available).

Conventions: linear weights are [out, in] (y = x W^T); no biases except optional frozen ones on q, k, v ("bq", "bk",
"bv" in the weight dict: the Qwen2.5 family the paper also evaluates, Sec. 8.1); A is [in, r],
B is [r, out]; `kv_len` counts tokens cached BEFORE the step (the step appends
one and attends over kv_len + 1).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F = np.float64


# =============================================================================
# element-wise pieces
# =============================================================================
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """h = x * g / sqrt(mean_j x_j^2 + eps), over the last axis."""
    x = np.asarray(x, F)
    rho = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * rho * np.asarray(g, F)


def rope_angles(pos: np.ndarray, d: int, base: float) -> np.ndarray:
    """angle[p, i] = pos_p * base^(-2 i / d), i < d/2."""
    i = np.arange(d // 2, dtype=F)
    theta = np.asarray(base, F) ** (-2.0 * i / d)
    return np.asarray(pos, F)[..., None] * theta


def rope(t: np.ndarray, pos: np.ndarray, base: float, inverse: bool = False) -> np.ndarray:
    """Rotary embedding with half-split pairs (i, i + d/2).

    t is [..., heads, d] and pos has the shape of the leading axes.
    (t_i, t_{i+d/2}) -> (t_i cos - t_{i+d/2} sin, t_{i+d/2} cos + t_i sin);
    `inverse` rotates by the negative angle (used by the backward pass).
    """
    t = np.asarray(t, F)
    d = t.shape[-1]
    ang = rope_angles(pos, d, base)[..., None, :]        # broadcast over heads
    c, s = np.cos(ang), np.sin(ang)
    if inverse:
        s = -s
    lo, hi = t[..., : d // 2], t[..., d // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def sigmoid(a: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-np.asarray(a, F)))


def silu(a: np.ndarray) -> np.ndarray:
    """silu(a) = a * sigmoid(a)."""
    return np.asarray(a, F) * sigmoid(a)


def softmax(s: np.ndarray) -> np.ndarray:
    """exp(s - max s) / sum, over the last axis."""
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def lora_linear(x: np.ndarray, W: np.ndarray, ab: Optional[Tuple[np.ndarray, np.ndarray]], scale: float):
    """y = x W^T + scale * (x A) B   (second term only if the projection is adapted)."""
    x = np.asarray(x, F)
    y = x @ np.asarray(W, F).T
    if ab is not None:
        A, B = np.asarray(ab[0], F), np.asarray(ab[1], F)
        y = y + scale * ((x @ A) @ B)
    return y


# =============================================================================
# attention, plain definition
# =============================================================================
def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query position over a run of cached tokens.

    q [n_q, d]; K, V [t, n_kv, d].  Query head j reads KV head j // (n_q/n_kv):
    s_t = q_j . K_{t,c} / sqrt(d);  p = softmax(s);  o_j = sum_t p_t V_{t,c}.
    """
    q, K, V = np.asarray(q, F), np.asarray(K, F), np.asarray(V, F)
    n_q, d = q.shape
    n_kv = K.shape[1]
    group = n_q // n_kv
    o = np.empty((n_q, d), F)
    for j in range(n_q):
        c = j // group
        s = (K[:, c, :] @ q[j]) / np.sqrt(F(d))
        p = softmax(s)
        o[j] = p @ V[:, c, :]
    return o


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray):
    """Full-sequence causal attention.  q [S, n_q, d], k/v [S, n_kv, d].

    Returns o [S, n_q, d] and the probabilities P [n_q, S, S] (row t attends
    columns 0..t) that the backward pass needs.
    """
    q, k, v = np.asarray(q, F), np.asarray(k, F), np.asarray(v, F)
    S, n_q, d = q.shape
    group = n_q // k.shape[1]
    mask = np.tril(np.ones((S, S), bool))
    P = np.zeros((n_q, S, S), F)
    o = np.empty((S, n_q, d), F)
    for j in range(n_q):
        c = j // group
        s = (q[:, j, :] @ k[:, c, :].T) / np.sqrt(F(d))
        s = np.where(mask, s, -np.inf)
        P[j] = softmax(s)
        o[:, j, :] = P[j] @ v[:, c, :]
    return o, P


# =============================================================================
# unified-pool geometry (Sec. 4.2: chunk = layerNum x 2 blocks; a column of the
# grid is the same token run in every layer's K and V)
# =============================================================================
@dataclass(frozen=True)
class PoolGeometry:
    block_bytes: int          # 2 MiB in the paper
    n_layers: int
    page_tokens: int          # 16-token pages
    kv_row_bytes: int         # one token's K (or V) in one layer
    small_pool_bytes: int     # the small-tensor pool sits at the start of the slab
    slab_bytes: int

    @property
    def page_bytes(self) -> int:
        return self.page_tokens * self.kv_row_bytes

    @property
    def pages_per_block(self) -> int:
        return self.block_bytes // self.page_bytes

    @property
    def chunk_bytes(self) -> int:
        return self.n_layers * 2 * self.block_bytes

    @property
    def n_chunks(self) -> int:
        return (self.slab_bytes - self.small_pool_bytes) // self.chunk_bytes

    def kv_offset(self, page: int, layer: int, kv: int) -> int:
        """Byte offset in the slab of page `page` of layer `layer`'s K (kv=0) or V (kv=1).

        page = chunk * pages_per_block + slot; inside a chunk block number
        2*layer + kv holds that layer's K or V, and the slot-th page of every
        block of the chunk belongs to the same 16 tokens.
        """
        chunk, slot = divmod(int(page), self.pages_per_block)
        return (self.small_pool_bytes + chunk * self.chunk_bytes
                + (2 * layer + kv) * self.block_bytes + slot * self.page_bytes)

    def head_offset(self, page: int, layer: int, kv: int, head: int, slot_in_page: int, head_bytes: int) -> int:
        """Byte offset of one token's vector of one KV head.  Inside a page the
        order is [kv head][token slot][head_dim]: the paper fixes the grid of
        pages, not the order inside an entry, and head-major keeps the 16
        tokens of one head contiguous."""
        return self.kv_offset(page, layer, kv) + (head * self.page_tokens + slot_in_page) * head_bytes


class PagedKV:
    """A paged cache over a flat element array (the 'slab'), read and written
    only through PoolGeometry's address function."""

    def __init__(self, geom: PoolGeometry, elem_bytes: int, n_kv: int, d: int,
                 slab: Optional[np.ndarray] = None):
        self.g, self.eb, self.n_kv, self.d = geom, elem_bytes, n_kv, d
        assert geom.kv_row_bytes == n_kv * d * elem_bytes
        self.slab = np.zeros(geom.slab_bytes // elem_bytes, F) if slab is None else slab

    def _vec(self, page: int, layer: int, kv: int, head: int, slot: int) -> slice:
        off = self.g.head_offset(page, layer, kv, head, slot, self.d * self.eb)
        assert off % self.eb == 0
        e = off // self.eb
        return slice(e, e + self.d)

    def write(self, table_row: Sequence[int], layer: int, pos: int, k: np.ndarray, v: np.ndarray):
        P = self.g.page_tokens
        page, slot = int(table_row[pos // P]), pos % P
        k, v = np.asarray(k, F).reshape(self.n_kv, self.d), np.asarray(v, F).reshape(self.n_kv, self.d)
        for c in range(self.n_kv):
            self.slab[self._vec(page, layer, 0, c, slot)] = k[c]
            self.slab[self._vec(page, layer, 1, c, slot)] = v[c]

    def gather(self, table_row: Sequence[int], layer: int, n: int):
        """K, V [n, n_kv, d] of logical positions 0..n-1."""
        P = self.g.page_tokens
        K = np.empty((n, self.n_kv, self.d), F)
        V = np.empty((n, self.n_kv, self.d), F)
        for t in range(n):
            page, slot = int(table_row[t // P]), t % P
            for c in range(self.n_kv):
                K[t, c] = self.slab[self._vec(page, layer, 0, c, slot)]
                V[t, c] = self.slab[self._vec(page, layer, 1, c, slot)]
        return K, V


# =============================================================================
# decode step (Sec. 2.1: one new token per sequence, reusing the cache)
# =============================================================================
@dataclass
class Shapes:
    hidden: int
    n_q: int
    n_kv: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0


def _bias(W, name):
    """Frozen additive bias of a projection (q, k, v of models that carry them), or 0.  It is added before the
    rotary embedding; being constant it receives no gradient and changes no other gradient formula."""
    b = W.get(name)
    return F(0.0) if b is None else np.asarray(b, F)


def _qkv_new_token(x, W, sh: Shapes, pos):
    """Steps 1-3 of the decode layer for one batch of single tokens."""
    h = rmsnorm(x, W["g1"], sh.rms_eps)
    B = h.shape[0]
    q = (h @ np.asarray(W["wq"], F).T + _bias(W, "bq")).reshape(B, sh.n_q, sh.head_dim)
    k = (h @ np.asarray(W["wk"], F).T + _bias(W, "bk")).reshape(B, sh.n_kv, sh.head_dim)
    v = (h @ np.asarray(W["wv"], F).T + _bias(W, "bv")).reshape(B, sh.n_kv, sh.head_dim)
    q = rope(q, pos, sh.rope_base)
    k = rope(k, pos, sh.rope_base)
    return q, k, v


def _post_attention(x, o, W, sh: Shapes):
    """x1 = x + o Wo^T;  y = x1 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T,  h2 = RMSNorm(x1)."""
    B = x.shape[0]
    x1 = np.asarray(x, F) + o.reshape(B, -1) @ np.asarray(W["wo"], F).T
    h2 = rmsnorm(x1, W["g2"], sh.rms_eps)
    a = h2 @ np.asarray(W["wg"], F).T
    u = h2 @ np.asarray(W["wu"], F).T
    m = silu(a) * u
    return x1 + m @ np.asarray(W["wd"], F).T


def decode_layer_contiguous(x: np.ndarray, W: Dict[str, np.ndarray], sh: Shapes,
                            cache: List[Tuple[np.ndarray, np.ndarray]]):
    """One decoder layer, one new token per sequence, contiguous cache.

    x [B, H]; cache[b] = (K, V) each [n_b, n_kv, d] (keys already rotated).
    Returns y [B, H] and the cache with the new token appended at position n_b.
    Decode uses base weights only (the finetune instance owns the adapters).
    """
    x = np.asarray(x, F)
    pos = np.array([c[0].shape[0] for c in cache])
    q, k, v = _qkv_new_token(x, W, sh, pos)
    new_cache, o = [], np.empty((x.shape[0], sh.n_q, sh.head_dim), F)
    for b, (K, V) in enumerate(cache):
        K2 = np.concatenate([np.asarray(K, F), k[b][None]], axis=0)
        V2 = np.concatenate([np.asarray(V, F), v[b][None]], axis=0)
        o[b] = attend(q[b], K2, V2)
        new_cache.append((K2, V2))
    return _post_attention(x, o, W, sh), new_cache


def decode_layer_paged(x: np.ndarray, W: Dict[str, np.ndarray], sh: Shapes, kv: PagedKV,
                       layer: int, kv_len: np.ndarray, page_table: np.ndarray):
    """Same layer over the paged cache: the new token is written to page
    table[b][n_b // P], slot n_b % P, then positions 0..n_b are read back
    through the page table.  Mutates `kv.slab`."""
    x = np.asarray(x, F)
    q, k, v = _qkv_new_token(x, W, sh, np.asarray(kv_len))
    o = np.empty((x.shape[0], sh.n_q, sh.head_dim), F)
    for b in range(x.shape[0]):
        n = int(kv_len[b])
        kv.write(page_table[b], layer, n, k[b], v[b])
        K, V = kv.gather(page_table[b], layer, n + 1)
        o[b] = attend(q[b], K, V)
    return _post_attention(x, o, W, sh)


def decode_model_paged(tokens_or_x, layers: List[Dict[str, np.ndarray]], extras: Optional[Dict[str, np.ndarray]],
                       sh: Shapes, kv: PagedKV, kv_len, page_table):
    """Embedding -> L layers -> final RMSNorm -> output layer (Sec. 2.1).

    With `extras` None the input is the hidden state and the hidden state after
    the last layer is returned; otherwise the input is token ids and
    (hidden, logits, argmax with ties to the lowest index) is returned.
    """
    if extras is None:
        x = np.asarray(tokens_or_x, F)
    else:
        x = np.asarray(extras["emb"], F)[np.asarray(tokens_or_x)]
    for l, W in enumerate(layers):
        x = decode_layer_paged(x, W, sh, kv, l, kv_len, page_table)
    if extras is None:
        return x
    h = rmsnorm(x, extras["gf"], sh.rms_eps)
    logits = h @ np.asarray(extras["wlm"], F).T
    return x, logits, np.argmax(logits, axis=-1)


# =============================================================================
# finetune layer: forward and backward (Sec. 6.1 unit: one layer x one micro-batch)
# =============================================================================
def layer_forward(X: np.ndarray, W: Dict[str, np.ndarray], lora: Dict[str, Tuple[np.ndarray, np.ndarray]],
                  scale: float, sh: Shapes):
    """Causal forward of one layer over X [B_f, S, H] with LoRA on the adapted
    projections.  Returns Y and everything the backward pass needs."""
    X = np.asarray(X, F)
    Bf, S, H = X.shape
    pos = np.broadcast_to(np.arange(S), (Bf, S))
    h = rmsnorm(X, W["g1"], sh.rms_eps)
    q0 = (lora_linear(h, W["wq"], lora.get("q"), scale) + _bias(W, "bq")).reshape(Bf, S, sh.n_q, sh.head_dim)
    k0 = (lora_linear(h, W["wk"], lora.get("k"), scale) + _bias(W, "bk")).reshape(Bf, S, sh.n_kv, sh.head_dim)
    v = (lora_linear(h, W["wv"], lora.get("v"), scale) + _bias(W, "bv")).reshape(Bf, S, sh.n_kv, sh.head_dim)
    q, k = rope(q0, pos, sh.rope_base), rope(k0, pos, sh.rope_base)
    o = np.empty((Bf, S, sh.n_q, sh.head_dim), F)
    P = []
    for b in range(Bf):
        o[b], Pb = causal_attention(q[b], k[b], v[b])
        P.append(Pb)
    of = o.reshape(Bf, S, -1)
    x1 = X + lora_linear(of, W["wo"], lora.get("o"), scale)
    h2 = rmsnorm(x1, W["g2"], sh.rms_eps)
    a = lora_linear(h2, W["wg"], lora.get("gate"), scale)
    u = lora_linear(h2, W["wu"], lora.get("up"), scale)
    m = silu(a) * u
    Y = x1 + lora_linear(m, W["wd"], lora.get("down"), scale)
    saved = dict(X=X, h=h, q=q, k=k, v=v, P=P, of=of, x1=x1, h2=h2, a=a, u=u, m=m)
    return Y, saved


def _rmsnorm_bwd(dy, x, g, eps):
    """With rho = (mean x^2 + eps)^(-1/2), xh = x rho:
    dx = rho * (dy*g - xh * mean(dy*g*xh))."""
    rho = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    xh = x * rho
    dyg = dy * np.asarray(g, F)
    return rho * (dyg - xh * np.mean(dyg * xh, axis=-1, keepdims=True))


def _linear_bwd(dy, xin, Wm, ab, scale, grads, name):
    """dx = dy W (+ scale (dy B^T) A^T);  dA += scale x^T (dy B^T);  dB += scale (x A)^T dy.
    The frozen W gets no gradient."""
    dx = dy @ np.asarray(Wm, F)
    if ab is not None:
        A, B = np.asarray(ab[0], F), np.asarray(ab[1], F)
        x2, dy2 = xin.reshape(-1, xin.shape[-1]), dy.reshape(-1, dy.shape[-1])
        g = dy2 @ B.T
        dx = dx + scale * (g @ A.T).reshape(dx.shape)
        dA = scale * (x2.T @ g)
        dB = scale * ((x2 @ A).T @ dy2)
        grads[name] = (dA, dB)
    return dx


def layer_backward(dY: np.ndarray, saved: dict, W: Dict[str, np.ndarray],
                   lora: Dict[str, Tuple[np.ndarray, np.ndarray]], scale: float, sh: Shapes):
    """Chain rule through the layer.  Returns dX and {proj: (dA, dB)}."""
    dY = np.asarray(dY, F)
    s = saved
    Bf, S, H = dY.shape
    grads: Dict[str, Tuple[np.ndarray, np.ndarray]] = {}
    # FFN
    dm = _linear_bwd(dY, s["m"], W["wd"], lora.get("down"), scale, grads, "down")
    sg = sigmoid(s["a"])
    da = dm * s["u"] * sg * (1.0 + s["a"] * (1.0 - sg))
    du = dm * s["a"] * sg
    dh2 = (_linear_bwd(da, s["h2"], W["wg"], lora.get("gate"), scale, grads, "gate")
           + _linear_bwd(du, s["h2"], W["wu"], lora.get("up"), scale, grads, "up"))
    dx1 = dY + _rmsnorm_bwd(dh2, s["x1"], W["g2"], sh.rms_eps)
    # attention output projection
    do = _linear_bwd(dx1, s["of"], W["wo"], lora.get("o"), scale, grads, "o")
    do = do.reshape(Bf, S, sh.n_q, sh.head_dim)
    # attention: dV = P^T dO, dP = dO V^T, dS = P*(dP - rowsum(dP*P)), dQ = dS K/sqrt(d), dK = dS^T Q/sqrt(d)
    group = sh.n_q // sh.n_kv
    dq = np.zeros_like(s["q"])
    dk = np.zeros_like(s["k"])
    dv = np.zeros_like(s["v"])
    inv = 1.0 / np.sqrt(F(sh.head_dim))
    for b in range(Bf):
        for j in range(sh.n_q):
            c = j // group
            Pj = s["P"][b][j]
            doj = do[b, :, j, :]
            dv[b, :, c, :] += Pj.T @ doj
            dP = doj @ s["v"][b, :, c, :].T
            dS = Pj * (dP - np.sum(dP * Pj, axis=-1, keepdims=True))
            dq[b, :, j, :] = dS @ s["k"][b, :, c, :] * inv
            dk[b, :, c, :] += dS.T @ s["q"][b, :, j, :] * inv
    pos = np.broadcast_to(np.arange(S), (Bf, S))
    dq0 = rope(dq, pos, sh.rope_base, inverse=True).reshape(Bf, S, -1)
    dk0 = rope(dk, pos, sh.rope_base, inverse=True).reshape(Bf, S, -1)
    dvf = dv.reshape(Bf, S, -1)
    dh = (_linear_bwd(dq0, s["h"], W["wq"], lora.get("q"), scale, grads, "q")
          + _linear_bwd(dk0, s["h"], W["wk"], lora.get("k"), scale, grads, "k")
          + _linear_bwd(dvf, s["h"], W["wv"], lora.get("v"), scale, grads, "v"))
    dX = dx1 + _rmsnorm_bwd(dh, s["X"], W["g1"], sh.rms_eps)
    return dX, grads


# =============================================================================
# losses (harness side)
# =============================================================================
def mse_loss(Y: np.ndarray, T: np.ndarray):
    """l = mean((Y - T)^2) over every element; dY = 2 (Y - T) / numel."""
    Y, T = np.asarray(Y, F), np.asarray(T, F)
    diff = Y - T
    return float(np.mean(diff * diff)), 2.0 * diff / diff.size


def ce_loss(logits: np.ndarray, targets: np.ndarray):
    """Mean negative log-likelihood of `targets` [N] under `logits` [N, V];
    d logits = (softmax - onehot) / N."""
    z = np.asarray(logits, F)
    N = z.shape[0]
    zmax = np.max(z, axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.sum(np.exp(z - zmax), axis=-1))
    loss = float(np.mean(lse - z[np.arange(N), targets]))
    d = softmax(z)
    d[np.arange(N), targets] -= 1.0
    return loss, d / N


def head_forward_backward(x: np.ndarray, g_final: np.ndarray, w_lm: np.ndarray, targets: np.ndarray, eps: float):
    """Output layer of the finetune task (Sec. 2.1: "output layer" after the stack of transformer layers) with the
    next-token cross entropy of the workloads that carry a vocabulary.

    x [N, H]: hidden states after the last layer; h = RMSNorm(x; g_final); logits = h W_lm^T  ([N, V]).
    targets [N]: class index per position, or -1 for a position that is not counted (the last token of a sequence).
    loss = mean over counted positions of -log softmax(logits)[target]; returns (loss, d loss / d x, logits).
    W_lm and g_final are frozen (no gradient)."""
    x = np.asarray(x, F)
    W = np.asarray(w_lm, F)
    t = np.asarray(targets)
    h = rmsnorm(x, g_final, eps)
    logits = h @ W.T
    valid = t >= 0
    n = int(valid.sum())
    loss, dl = ce_loss(logits[valid], t[valid])          # dl = (softmax - onehot) / n over the counted rows
    dlogits = np.zeros_like(logits)
    dlogits[valid] = dl
    dh = dlogits @ W
    dx = _rmsnorm_bwd(dh, x, g_final, eps)
    return loss, dx, logits
