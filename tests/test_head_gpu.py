"""GPU parity of harli_head_fwd_bwd (output layer + next-token cross entropy) and of a whole-model finetune step
(embedding -> layers -> output layer -> loss -> backward through every layer) against the CPU oracle."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import harli_oracle as O
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import assert_close, f32_dev, shapes_of, to_dev

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class ModelCase:
    """A small multi-layer model with a vocabulary, adapters on every layer, and a token micro-batch."""

    def __init__(self, n_layers=2, vocab=1000, micro_batch=2, seq_len=96, **model_kw):
        w = wl.workload(0)
        m = dataclasses.replace(w.model, dtype="bf16", n_layers=n_layers, vocab=vocab, **model_kw)
        self.w, self.m = dataclasses.replace(w, model=m), m
        self.lora = wl.LoraCfg(8, 16.0, ("q", "k", "v", "o"))
        self.Bf, self.S = micro_batch, seq_len
        T = micro_batch * seq_len
        self.T = T
        self.layers_np = [wl.make_layer_weights(self.w, l, m) for l in range(n_layers)]
        self.lora_np = [wl.make_lora(self.w, l, m, self.lora) for l in range(n_layers)]
        self.ex = wl.make_model_extras(self.w, m)
        self.tok = wl.make_token_ids(self.w, (micro_batch, seq_len))
        # next-token targets: position t predicts token t+1; the last position of each sequence is not counted
        tg = np.full((micro_batch, seq_len), -1, np.int32)
        tg[:, :-1] = self.tok[:, 1:]
        self.targets = tg
        block = 2 << 20
        chunk = n_layers * 2 * block
        slab_bytes = (8 << 20) + 24 * chunk
        self.slab = torch.zeros(slab_bytes, dtype=torch.uint8, device=DEV)
        self.pool = hb.Pool(self.slab, slab_bytes, block_bytes=block, n_layers=n_layers, kv_row_bytes=m.kv_row_bytes,
                            small_pool_bytes=8 << 20, kv_reserve_chunks=1)
        self.layers_dev = []
        for L in self.layers_np:
            dl = {n: to_dev(L[n], "bf16") for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")}
            dl["g1"], dl["g2"] = f32_dev(L["g1"]), f32_dev(L["g2"])
            for bn in ("bq", "bk", "bv"):
                if bn in L:
                    dl[bn] = f32_dev(L[bn])
            self.layers_dev.append(dl)
        self.emb_dev, self.gf_dev, self.wlm_dev = to_dev(self.ex["emb"], "bf16"), f32_dev(self.ex["gf"]), to_dev(self.ex["wlm"], "bf16")
        self.ctx = hb.Context(self.pool, n_layers=n_layers, hidden=m.hidden, n_q_heads=m.n_q, n_kv_heads=m.n_kv,
                              head_dim=m.head_dim, ffn=m.ffn, vocab=vocab, rms_eps=m.rms_eps, rope_base=m.rope_base,
                              dtype=hb.HARLI_BF16, max_batch=1, max_seq_len=16, max_ft_tokens=T, layers=self.layers_dev,
                              emb=self.emb_dev, g_final=self.gf_dev, w_lm=self.wlm_dev)
        self.A_dev = [{p: to_dev(a, "bf16") for p, (a, b) in ln.items()} for ln in self.lora_np]
        self.B_dev = [{p: to_dev(b, "bf16") for p, (a, b) in ln.items()} for ln in self.lora_np]
        self.ctx.lora_attach(self.lora.rank, self.lora.alpha, self.lora.targets, self.A_dev, self.B_dev)


@pytest.mark.parametrize("vocab,T", [(1000, 192), (777, 130), (4096, 64)])
def test_head_loss_and_dx_match_the_oracle(vocab, T):
    """Vocabulary sizes with and without padding to a multiple of 8, some positions not counted."""
    case = ModelCase(n_layers=1, vocab=vocab, micro_batch=1, seq_len=200)
    rng = np.random.default_rng(vocab)
    x = rng.standard_normal((T, case.m.hidden)).astype(np.float32) * 1.5
    tg = rng.integers(0, vocab, size=T).astype(np.int32)
    tg[rng.random(T) < 0.2] = -1
    loss = torch.zeros(1, device=DEV)
    dx = torch.empty(T, case.m.hidden, device=DEV)
    case.ctx.head_fwd_bwd(f32_dev(x), torch.from_numpy(tg).to(DEV), loss, dx)
    torch.cuda.synchronize()
    case.ctx.check()
    ref_loss, ref_dx, _ = O.head_forward_backward(x, case.ex["gf"], case.ex["wlm"], tg, case.m.rms_eps)
    assert abs(float(loss) - ref_loss) <= 2e-3 * abs(ref_loss), (float(loss), ref_loss)
    assert_close(dx.cpu().numpy(), ref_dx, "head dx")
    # the rows' losses are added in a fixed order: the same bits on every call
    loss2, dx2 = torch.zeros(1, device=DEV), torch.empty_like(dx)
    for _ in range(3):
        case.ctx.head_fwd_bwd(f32_dev(x), torch.from_numpy(tg).to(DEV), loss2, dx2)
        torch.cuda.synchronize()
        assert torch.equal(loss, loss2) and torch.equal(dx, dx2)
    # an out-of-range class is reported, not dereferenced
    tg[0] = vocab + 5
    case.ctx.head_fwd_bwd(f32_dev(x), torch.from_numpy(tg).to(DEV), loss, dx)
    torch.cuda.synchronize()
    with pytest.raises(hb.HarliError):
        case.ctx.check()


def test_whole_model_finetune_step_matches_the_oracle():
    """Two layers with adapters, vocabulary 1000, 2 x 96 tokens: loss, the gradient reaching the embedding output and
    every adapter gradient of both layers."""
    case = ModelCase(n_layers=2, vocab=1000, micro_batch=2, seq_len=96)
    m, T, H = case.m, case.T, case.m.hidden
    sh = shapes_of(m)
    x0 = case.ex["emb"][case.tok.reshape(-1)].astype(np.float32)           # embedding gather (host side of the harness)
    # ---- GPU
    xs = [f32_dev(x0)]
    saved = []
    for l in range(2):
        y = torch.empty(T, H, dtype=torch.float32, device=DEV)
        saved.append(case.ctx.lora_fwd(l, xs[-1], y, case.Bf, case.S))
        xs.append(y)
    loss = torch.zeros(1, device=DEV)
    d = torch.empty(T, H, device=DEV)
    case.ctx.head_fwd_bwd(xs[-1], torch.from_numpy(case.targets.reshape(-1)).to(DEV), loss, d)
    grads_gpu = []
    for l in (1, 0):
        dA = {p: torch.zeros(a.shape, dtype=torch.float32, device=DEV) for p, (a, b) in case.lora_np[l].items()}
        dB = {p: torch.zeros(b.shape, dtype=torch.float32, device=DEV) for p, (a, b) in case.lora_np[l].items()}
        dprev = torch.empty(T, H, device=DEV)
        case.ctx.lora_bwd(l, d, dprev, saved[l], dA, dB)
        grads_gpu.insert(0, (dA, dB))
        d = dprev
    torch.cuda.synchronize()
    case.ctx.check()
    # ---- oracle
    X = x0.reshape(case.Bf, case.S, H)
    acts, svs = [X], []
    for l in range(2):
        Y, sv = O.layer_forward(acts[-1], case.layers_np[l], case.lora_np[l], case.lora.scale, sh)
        acts.append(Y)
        svs.append(sv)
    ref_loss, dlast, _ = O.head_forward_backward(acts[-1].reshape(T, H), case.ex["gf"], case.ex["wlm"], case.targets.reshape(-1), m.rms_eps)
    dref = dlast.reshape(case.Bf, case.S, H)
    grads_ref = [None, None]
    for l in (1, 0):
        dref, grads_ref[l] = O.layer_backward(dref, svs[l], case.layers_np[l], case.lora_np[l], case.lora.scale, sh)
    print("loss GPU %.6f oracle %.6f" % (float(loss), ref_loss))
    assert abs(float(loss) - ref_loss) <= 2e-3 * abs(ref_loss)
    assert_close(d.cpu().numpy().reshape(dref.shape), dref, "gradient at the embedding output")
    for l in range(2):
        for p in grads_ref[l]:
            assert_close(grads_gpu[l][0][p].cpu().numpy(), grads_ref[l][p][0], "layer %d dA[%s]" % (l, p))
            assert_close(grads_gpu[l][1][p].cpu().numpy(), grads_ref[l][p][1], "layer %d dB[%s]" % (l, p))
    st = case.pool.stats()
    assert st.tensor_blocks_live == 0 and st.small_bytes_live == 0
