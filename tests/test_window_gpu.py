"""Window over the finetune task's frozen weights on the device (Sec. 4.3): a whole-model training step gives
bit-identical results with every window size, after a resize and after the window is removed; the copies follow the
model's plan (hits, refills, bytes); an out-of-order call is served on demand; the result matches the oracle."""
import numpy as np
import pytest
import torch

from oracle import harli_oracle as O
from oracle import window_model as WM
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import assert_close, f32_dev, shapes_of
from tests.test_head_gpu import DEV, ModelCase

pytestmark = pytest.mark.gpu

L = 4


def run_step(case):
    m, T, H = case.m, case.T, case.m.hidden
    x0 = case.ex["emb"][case.tok.reshape(-1)].astype(np.float32)
    xs, saved = [f32_dev(x0)], []
    for l in range(L):
        y = torch.empty(T, H, dtype=torch.float32, device=DEV)
        saved.append(case.ctx.lora_fwd(l, xs[-1], y, case.Bf, case.S))
        xs.append(y)
    loss = torch.zeros(1, device=DEV)
    d = torch.empty(T, H, device=DEV)
    case.ctx.head_fwd_bwd(xs[-1], torch.from_numpy(case.targets.reshape(-1)).to(DEV), loss, d)
    grads = []
    for l in range(L - 1, -1, -1):
        dA = {p: torch.zeros(a.shape, dtype=torch.float32, device=DEV) for p, (a, b) in case.lora_np[l].items()}
        dB = {p: torch.zeros(b.shape, dtype=torch.float32, device=DEV) for p, (a, b) in case.lora_np[l].items()}
        dprev = torch.empty(T, H, device=DEV)
        case.ctx.lora_bwd(l, d, dprev, saved[l], dA, dB)
        grads.insert(0, (dA, dB))
        d = dprev
    torch.cuda.synchronize()
    case.ctx.check()
    return loss, d, grads, xs[-1]


def same(a, b):
    la, da, ga, ya = a
    lb, db, gb, yb = b
    # the loss is a sum of per-row terms by float atomics (order varies); everything else has a fixed order
    if abs(float(la) - float(lb)) > 1e-5 * abs(float(lb)) or not (torch.equal(da, db) and torch.equal(ya, yb)):
        return False
    return all(torch.equal(ga[l][k][p], gb[l][k][p]) for l in range(L) for k in (0, 1) for p in ga[l][k])


def test_training_step_is_bit_identical_under_every_window():
    case = ModelCase(n_layers=L, vocab=1000, micro_batch=2, seq_len=96)
    base = run_step(case)
    assert case.ctx.ft_window_stats().slots == 0 and case.ctx.ft_window_ready(3, True)
    free0 = case.pool.stats().tensor_blocks_live
    for n in (1, 2, 3, 5, 6, 7, 8, 50):
        case.ctx.ft_window_enable(n)
        st0 = case.ctx.ft_window_stats()
        n_eff = min(n, 2 * L)
        assert st0.slots == n_eff and st0.host_bytes == 2 * L * st0.slot_bytes and st0.h2d_bytes == n_eff * st0.slot_bytes
        assert case.pool.stats().tensor_blocks_live > free0                 # the slots come from the unified pool
        torch.cuda.synchronize()
        assert case.ctx.ft_window_ready(0, False)
        assert case.ctx.ft_window_ready(L - 1, True) == (WM.item_of(L - 1, True, L) in WM.wanted_items(L, n_eff))   # as the model places them
        for rep in range(2):
            assert same(run_step(case), base), "window of %d slots, step %d" % (n, rep)
        st = case.ctx.ft_window_stats()
        assert st.hits == 4 * L and st.misses == 0
        model = WM.Window(L, n_eff)                                          # the copies follow the model's plan
        want_refills = sum(model.access(it)[2] >= 0 for it in list(range(2 * L)) * 2)
        assert st.refills == want_refills and (want_refills == 4 * L) == (n_eff <= WM.LOOKAHEAD)
        assert st.h2d_bytes == (n_eff + st.refills) * st.slot_bytes
        with pytest.raises(hb.HarliError) as e:
            case.ctx.ft_window_enable(2)
        assert e.value.status == hb.HARLI_ERR_STATE
        case.ctx.ft_window_disable()
        assert case.pool.stats().tensor_blocks_live == free0
    assert same(run_step(case), base)                                       # back on copies of its own
    with pytest.raises(hb.HarliError):
        case.ctx.ft_window_disable()


def test_resize_and_out_of_order_calls():
    case = ModelCase(n_layers=L, vocab=1000, micro_batch=2, seq_len=96)
    base = run_step(case)
    case.ctx.ft_window_enable(3)
    assert same(run_step(case), base)
    case.ctx.ft_window_resize(1)                                             # memory pressure: shrink (Sec. 4.4)
    assert case.ctx.ft_window_stats().slots == 1
    assert same(run_step(case), base)
    case.ctx.ft_window_resize(6)
    assert case.ctx.ft_window_stats().slots == 6
    assert same(run_step(case), base)
    m0 = case.ctx.ft_window_stats().misses
    # a forward pass of layer 2 alone, out of the regular order: loaded on demand, same output as in the regular walk
    T, H = case.T, case.m.hidden
    x0 = case.ex["emb"][case.tok.reshape(-1)].astype(np.float32)
    xs = [f32_dev(x0)]
    for l in range(2):
        y = torch.empty(T, H, dtype=torch.float32, device=DEV)
        case.ctx.saved_release(case.ctx.lora_fwd(l, xs[-1], y, case.Bf, case.S))
        xs.append(y)
    case.ctx.ft_window_resize(1)
    y2 = torch.empty(T, H, dtype=torch.float32, device=DEV)
    case.ctx.saved_release(case.ctx.lora_fwd(2, xs[-1], y2, case.Bf, case.S))
    y2b = torch.empty(T, H, dtype=torch.float32, device=DEV)
    case.ctx.saved_release(case.ctx.lora_fwd(2, xs[-1], y2b, case.Bf, case.S))   # again: the copy was evicted after use
    torch.cuda.synchronize()
    assert torch.equal(y2, y2b)
    assert case.ctx.ft_window_stats().misses >= m0 + 1
    assert same(run_step(case), base)


def test_a_pool_without_room_refuses_the_window_and_keeps_the_copies():
    case = ModelCase(n_layers=L, vocab=1000, micro_batch=2, seq_len=96)
    base = run_step(case)
    held = []
    chunk = L * 2 * (2 << 20)
    while True:                                                             # fill the pool with chunk-sized tensors
        try:
            held.append(case.pool.alloc(hb.CLS_TENSOR, chunk))
        except hb.HarliError:
            break
    with pytest.raises(hb.HarliError) as e:
        case.ctx.ft_window_enable(2)
    assert e.value.status == hb.HARLI_ERR_OOM
    assert case.ctx.ft_window_stats().slots == 0
    for a in held:
        case.pool.free(a)
    assert same(run_step(case), base)                                       # nothing was moved


def test_windowed_step_matches_the_oracle():
    case = ModelCase(n_layers=L, vocab=1000, micro_batch=2, seq_len=96)
    case.ctx.ft_window_enable(2)
    loss, d, grads, _ = run_step(case)
    m, T, H = case.m, case.T, case.m.hidden
    sh = shapes_of(m)
    x0 = case.ex["emb"][case.tok.reshape(-1)].astype(np.float32)
    acts, svs = [x0.reshape(case.Bf, case.S, H)], []
    for l in range(L):
        Y, sv = O.layer_forward(acts[-1], case.layers_np[l], case.lora_np[l], case.lora.scale, sh)
        acts.append(Y)
        svs.append(sv)
    ref_loss, dlast, _ = O.head_forward_backward(acts[-1].reshape(T, H), case.ex["gf"], case.ex["wlm"], case.targets.reshape(-1), m.rms_eps)
    dref = dlast.reshape(case.Bf, case.S, H)
    gref = [None] * L
    for l in range(L - 1, -1, -1):
        dref, gref[l] = O.layer_backward(dref, svs[l], case.layers_np[l], case.lora_np[l], case.lora.scale, sh)
    assert abs(float(loss) - ref_loss) <= 2e-3 * abs(ref_loss)
    assert_close(d.cpu().numpy().reshape(dref.shape), dref, "gradient at the embedding output")
    for l in range(L):
        for p in gref[l]:
            assert_close(grads[l][0][p].cpu().numpy(), gref[l][p][0], "layer %d dA[%s]" % (l, p))
            assert_close(grads[l][1][p].cpu().numpy(), gref[l][p][1], "layer %d dB[%s]" % (l, p))
