"""Shapes and seeded random inputs of the synthetic workloads.

The five workloads mirror the configurations the build is measured on: a tiny
fp32 layer, a 7B-class layer, the 32-layer 7B-class model, a 13B-class model
and an 8B-class GQA model.  They stand in for the paper's LLaMA3-8B /
Qwen2.5-7B checkpoints, its production request trace and its (unnamed)
finetune dataset, none of which are available: every tensor is drawn from a
counter-based generator (Philox) keyed by ``1000 * config + stream`` and, for
per-layer tensors, the layer index, so the oracle tests and the HIP path see
the same bytes.

Nothing in this file computes any part of the method; it only draws numbers,
rounds them to the storage type and describes shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

LORA_TARGETS = ("q", "k", "v", "o", "gate", "up", "down")
WEIGHT_NAME = dict(q="wq", k="wk", v="wv", o="wo", gate="wg", up="wu", down="wd")

# random streams (second term of the seed)
S_WEIGHTS, S_ADAPTERS, S_INPUTS, S_TARGETS, S_LENGTHS, S_PAGES, S_ARRIVALS, S_KV = range(8)


@dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    hidden: int
    n_q: int
    n_kv: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    dtype: str = "bf16"          # storage type of weights, KV cache and saved activations
    qkv_bias: bool = False       # frozen additive biases on the q, k, v projections (the Qwen2.5 family)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def proj_shape(self, p: str) -> Tuple[int, int]:
        """(out_features, in_features) of projection ``p``; weights are [out, in]."""
        q, kv, h, f = self.n_q * self.head_dim, self.n_kv * self.head_dim, self.hidden, self.ffn
        return {"q": (q, h), "k": (kv, h), "v": (kv, h), "o": (h, q),
                "gate": (f, h), "up": (f, h), "down": (h, f)}[p]

    @property
    def layer_params(self) -> int:
        return sum(o * i for o, i in (self.proj_shape(p) for p in LORA_TARGETS))

    @property
    def kv_row_bytes(self) -> int:
        """Bytes of one token's K (or V) in one layer."""
        return self.n_kv * self.head_dim * self.elem_bytes


@dataclass(frozen=True)
class LoraCfg:
    rank: int
    alpha: float
    targets: Tuple[str, ...]

    @property
    def scale(self) -> float:
        return self.alpha / self.rank


@dataclass(frozen=True)
class DecodeCfg:
    batch: int
    len_dist: Tuple            # ("uniform", lo, hi) | ("const", n) | ("lognormal", median, sigma, cap)
    page_tokens: int = 16


@dataclass(frozen=True)
class FinetuneCfg:
    micro_batch: int
    seq_len: int
    loss: str = "mse"

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq_len


@dataclass(frozen=True)
class Workload:
    idx: int
    model: ModelCfg
    lora: LoraCfg
    decode: DecodeCfg
    finetune: FinetuneCfg
    batch_sweep: Tuple[int, ...] = field(default_factory=tuple)


CONFIGS: Dict[int, Workload] = {
    0: Workload(0, ModelCfg("tiny-fp32", 1, 256, 4, 4, 64, 688, 0, dtype="f32"),
                LoraCfg(8, 16.0, ("q", "v")),
                DecodeCfg(4, ("uniform", 64, 128)), FinetuneCfg(2, 128)),
    1: Workload(1, ModelCfg("7b-layer", 1, 4096, 32, 32, 128, 11008, 0),
                LoraCfg(16, 32.0, ("q", "k", "v", "o")),
                DecodeCfg(8, ("uniform", 256, 2048)), FinetuneCfg(4, 512)),
    2: Workload(2, ModelCfg("7b-32l", 32, 4096, 32, 32, 128, 11008, 32000),
                LoraCfg(16, 32.0, ("q", "k", "v", "o")),
                DecodeCfg(16, ("const", 1024)), FinetuneCfg(8, 512, "ce"),
                batch_sweep=(1, 4, 16, 64, 256)),
    3: Workload(3, ModelCfg("13b-40l", 40, 5120, 40, 40, 128, 13824, 32000),
                LoraCfg(64, 128.0, LORA_TARGETS),
                DecodeCfg(32, ("lognormal", 1200, 0.6, 4096)), FinetuneCfg(4, 1024, "ce")),
    4: Workload(4, ModelCfg("8b-gqa-32l", 32, 4096, 32, 8, 128, 14336, 128256),
                LoraCfg(32, 64.0, ("q", "k", "v", "o")),
                DecodeCfg(8, ("lognormal", 800, 0.6, 8192)), FinetuneCfg(8, 512, "ce")),
    # the second model family of the paper's evaluation (Sec. 8.1): a Qwen2.5-7B-class decoder -- 28 layers, hidden
    # 3584, 28 query heads over 4 KV heads (groups of 7), head_dim 128, ffn 18944, vocabulary 152064, RoPE base 1e6,
    # biases on q, k, v
    5: Workload(5, ModelCfg("qwen7b-class-28l", 28, 3584, 28, 4, 128, 18944, 152064, rope_base=1.0e6, qkv_bias=True),
                LoraCfg(16, 32.0, ("q", "k", "v", "o")),
                DecodeCfg(8, ("lognormal", 800, 0.6, 8192)), FinetuneCfg(8, 512, "ce")),
}


def workload(idx: int) -> Workload:
    return CONFIGS[idx]


# --------------------------------------------------------------------------- RNG
def rng_for(config: int, stream: int, sub: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (1000*config + stream, sub)."""
    return np.random.Generator(np.random.Philox(key=[1000 * config + stream, sub]))


# --------------------------------------------------------------------------- bf16 storage
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 values that are exactly representable in bfloat16."""
    return bf16_from_bits(bf16_bits(x)).reshape(np.shape(x))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32, copy=False)
    return bf16_round(x) if dtype == "bf16" else x


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return a


# --------------------------------------------------------------------------- tensors
def make_layer_weights(w: Workload, layer: int = 0, model: ModelCfg | None = None) -> Dict[str, np.ndarray]:
    """Frozen weights of one decoder layer: projections ~N(0, 0.02) stored as
    ``model.dtype``; RMSNorm gains 1 + 0.02*N(0,1) kept in float32; with ``qkv_bias`` the
    biases bq, bk, bv ~N(0, 0.5) in float32 (the same order of magnitude as the projections' outputs)."""
    m = model or w.model
    rng = rng_for(w.idx, S_WEIGHTS, layer)
    out = {}
    for p in LORA_TARGETS:
        out[WEIGHT_NAME[p]] = _store(_normal(rng, m.proj_shape(p), 0.02), m.dtype)
    out["g1"] = (1.0 + _normal(rng, (m.hidden,), 0.02)).astype(np.float32)
    out["g2"] = (1.0 + _normal(rng, (m.hidden,), 0.02)).astype(np.float32)
    if m.qkv_bias:                       # drawn last, so that models without biases keep their weights
        for p in ("q", "k", "v"):
            out["b" + p] = _normal(rng, (m.proj_shape(p)[0],), 0.5).astype(np.float32)
    return out


def make_model_extras(w: Workload, model: ModelCfg | None = None) -> Dict[str, np.ndarray]:
    """Embedding table, final gain and output layer of a full model."""
    m = model or w.model
    rng = rng_for(w.idx, S_WEIGHTS, 1_000_000)
    return {
        "emb": _store(_normal(rng, (m.vocab, m.hidden), 1.0), m.dtype),
        "gf": (1.0 + _normal(rng, (m.hidden,), 0.02)).astype(np.float32),
        "wlm": _store(_normal(rng, (m.vocab, m.hidden), 0.02), m.dtype),
    }


def make_lora(w: Workload, layer: int = 0, model: ModelCfg | None = None, lora: LoraCfg | None = None,
              zero_b: bool = False) -> Dict[str, Tuple[np.ndarray, np.ndarray]]:
    """Adapters of one layer: A [in, r] ~N(0, 1/8), B [r, out] ~N(0, 0.01)."""
    m, lc = model or w.model, lora or w.lora
    rng = rng_for(w.idx, S_ADAPTERS, layer)
    out = {}
    for p in LORA_TARGETS:           # draw for every target so a target subset does not shift the stream
        o, i = m.proj_shape(p)
        a = _store(_normal(rng, (i, lc.rank), 0.125), m.dtype)
        b = _store(_normal(rng, (lc.rank, o), 0.01), m.dtype)
        if p in lc.targets:
            out[p] = (a, np.zeros_like(b) if zero_b else b)
    return out


def draw_lengths(w: Workload, batch: int | None = None, dist: Tuple | None = None) -> np.ndarray:
    """Tokens already cached per sequence before the step."""
    d = dist or w.decode.len_dist
    b = batch or w.decode.batch
    rng = rng_for(w.idx, S_LENGTHS)
    if d[0] == "uniform":
        n = rng.integers(d[1], d[2] + 1, size=b)
    elif d[0] == "const":
        n = np.full(b, d[1])
    elif d[0] == "lognormal":
        z = rng.standard_normal(b)
        n = np.minimum(d[3], np.rint(np.exp(np.log(d[1]) + d[2] * z)))
    else:
        raise ValueError(d)
    return n.astype(np.int32)


def make_decode_inputs(w: Workload, batch: int | None = None, model: ModelCfg | None = None,
                       lengths: np.ndarray | None = None, n_layers: int | None = None):
    """Hidden-state input, cached lengths and cache contents of one decode step.

    Returns ``x`` [B, H] float32 ~N(0,1), ``kv_len`` [B] int32, and per layer a
    list over sequences of (K, V) arrays [n_b, n_kv, d] ~N(0,1) in the storage
    type (cached keys are taken as already rotated).
    """
    m = model or w.model
    b = batch or w.decode.batch
    kv_len = draw_lengths(w, b) if lengths is None else np.asarray(lengths, np.int32)
    x = _normal(rng_for(w.idx, S_INPUTS), (b, m.hidden), 1.0)
    layers = []
    for l in range(n_layers if n_layers is not None else m.n_layers):
        rng = rng_for(w.idx, S_KV, l)
        seqs = []
        for s in range(b):
            n = int(kv_len[s])
            k = _store(_normal(rng, (n, m.n_kv, m.head_dim), 1.0), m.dtype)
            v = _store(_normal(rng, (n, m.n_kv, m.head_dim), 1.0), m.dtype)
            seqs.append((k, v))
        layers.append(seqs)
    return x, kv_len, layers


def page_order(w: Workload, n_pages: int) -> np.ndarray:
    """Seeded permutation used to scatter logical pages over physical ones."""
    return rng_for(w.idx, S_PAGES).permutation(n_pages).astype(np.int64)


def make_finetune_inputs(w: Workload, model: ModelCfg | None = None, ft: FinetuneCfg | None = None):
    """Layer input X [B_f, S, H] ~N(0,1) and MSE target of the same shape."""
    m, f = model or w.model, ft or w.finetune
    x = _normal(rng_for(w.idx, S_INPUTS, 1), (f.micro_batch, f.seq_len, m.hidden), 1.0)
    tgt = _normal(rng_for(w.idx, S_TARGETS), (f.micro_batch, f.seq_len, m.hidden), 1.0)
    return x, tgt


def make_token_ids(w: Workload, shape) -> np.ndarray:
    m = w.model
    return rng_for(w.idx, S_INPUTS, 2).integers(0, m.vocab, size=shape).astype(np.int32)


def make_arrivals(w: Workload, steps: int, targets=(1, 8, 42, 24, 128, 256), mean_out: int = 256, phase_steps: int | None = None,
                  prompt=("lognormal", 800, 0.6, 8192)):
    """Request arrivals of a decode service, one list per decode step: [(prompt tokens, output tokens), ...].

    Piecewise-constant Poisson rate lambda(t) = target_batch / mean_out requests per step (Little's law: with a mean
    output length of `mean_out` steps that load settles at `target_batch` running sequences), the targets taken in
    turn for `phase_steps` steps each (default: steps / len(targets)); 8 / 42 / 24 are the light / heavy / medium loads
    of the paper's controlled experiment (Sec. 8.5).  Prompt lengths follow `prompt` (as `DecodeCfg.len_dist`), output
    lengths are geometric with mean `mean_out` on {1, 2, ...}.  Seeded by the workload index."""
    rng = rng_for(w.idx, S_ARRIVALS)
    ph = phase_steps or max(1, steps // len(targets))
    out = []
    for t in range(steps):
        lam = targets[(t // ph) % len(targets)] / float(mean_out)
        n = int(rng.poisson(lam))
        reqs = []
        for _ in range(n):
            if prompt[0] == "lognormal":
                pl = int(min(prompt[3], max(1, round(float(np.exp(np.log(prompt[1]) + prompt[2] * rng.standard_normal()))))))
            elif prompt[0] == "uniform":
                pl = int(rng.integers(prompt[1], prompt[2] + 1))
            else:
                pl = int(prompt[1])
            reqs.append((pl, int(rng.geometric(1.0 / mean_out))))
        out.append(reqs)
    return out
