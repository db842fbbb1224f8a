"""GPU parity of harli_adamw_step against the AdamW oracle, and of a short training run (forward, loss, backward,
update, repeated) against the same loop on the CPU oracle."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import harli_oracle as O
from oracle.optim_oracle import adamw_step
from paper_2511_11729_amd import binding as hb
from tests.gpu_util import FinetuneCase, f32_dev, shapes_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n", [1, 255, 4096 * 16 + 3])
def test_adamw_matches_the_oracle_over_several_steps(n):
    """fp32 kernel against the fp64 definition: relative 1e-5 on the parameters after 8 steps; the bf16 copy is the
    round-to-nearest-even of the kernel's own fp32 master, bit for bit."""
    rng = np.random.default_rng(n)
    p0 = rng.standard_normal(n).astype(np.float32)
    master, m, v = f32_dev(p0), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    param = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    p, mo, vo = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    kw = dict(lr=2e-3, beta1=0.9, beta2=0.98, eps=1e-7, weight_decay=0.05)
    for t in range(1, 9):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1)).astype(np.float32)
        grad = f32_dev(g)
        hb.adamw_step(master, m, v, grad, param, step=t, grad_scale=0.5, zero_grad=(t % 2 == 0), **kw)
        torch.cuda.synchronize()
        p, mo, vo = adamw_step(p, g, mo, vo, t, lr=2e-3, b1=0.9, b2=0.98, eps=1e-7, wd=0.05, grad_scale=0.5)
        assert bool((grad == 0).all()) == (t % 2 == 0)
    got = master.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - p)) <= 1e-5 * np.max(np.abs(p)) + 1e-7
    # moments: sums with cancellation -> absolute error relative to the largest entry
    assert np.max(np.abs(m.cpu().numpy() - mo)) <= 1e-5 * np.max(np.abs(mo)) + 1e-30
    assert np.max(np.abs(v.cpu().numpy() - vo)) <= 1e-5 * np.max(np.abs(vo)) + 1e-30
    want_bits = wl.bf16_bits(master.cpu().numpy())
    assert np.array_equal(param.view(torch.int16).cpu().numpy().view(np.uint16), want_bits)


def test_adamw_rejects_bad_arguments():
    x = torch.zeros(8, device=DEV)
    with pytest.raises(hb.HarliError):
        hb.adamw_step(x, x, x, x, None, step=0)
    with pytest.raises(hb.HarliError):
        hb.adamw_step(x, x, x, x, None, step=1, beta1=1.0)
    with pytest.raises(hb.HarliError):
        hb.adamw_step(x, x, x, None, None, step=1)


def test_training_run_follows_the_oracle():
    """Six updates of the adapters on config 0's shapes: both sides start from the same bf16 adapters, keep fp32 / fp64
    master copies, and feed the bf16-rounded adapters to the next forward pass.  The loss falls, and the two loss
    curves and the final adapters agree within the bf16 bar."""
    w = wl.workload(0)
    m = dataclasses.replace(w.model, dtype="bf16")
    case = FinetuneCase(w, m, w.lora, w.finetune)
    sh = shapes_of(m)
    T, H = case.ft.tokens, m.hidden
    kw = dict(lr=5e-3, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.0)
    # GPU state
    masters = {p: (case.A_dev[p].float().clone(), case.B_dev[p].float().clone()) for p in case.A_dev}
    mom = {p: tuple(torch.zeros_like(t) for t in (masters[p][0], masters[p][0], masters[p][1], masters[p][1])) for p in masters}
    dA = {p: torch.zeros_like(masters[p][0]) for p in masters}
    dB = {p: torch.zeros_like(masters[p][1]) for p in masters}
    Y = torch.empty(T, H, dtype=torch.float32, device=DEV)
    dX = torch.empty(T, H, dtype=torch.float32, device=DEV)
    Tg = case.T_np.reshape(T, H)
    # oracle state
    o_lora = {p: (a.astype(np.float64), b.astype(np.float64)) for p, (a, b) in case.lora_np.items()}
    o_mom = {p: [np.zeros_like(o_lora[p][0]), np.zeros_like(o_lora[p][0]), np.zeros_like(o_lora[p][1]), np.zeros_like(o_lora[p][1])]
             for p in o_lora}
    gpu_loss, ora_loss = [], []
    for t in range(1, 7):
        # ---- GPU: forward, loss on the host from the GPU's own Y, backward, update
        sv = case.ctx.lora_fwd(0, case.X_dev, Y, case.ft.micro_batch, case.ft.seq_len)
        y = Y.cpu().numpy().astype(np.float64)
        loss, dY = O.mse_loss(y.reshape(case.X_np.shape), case.T_np)
        gpu_loss.append(loss)
        case.ctx.lora_bwd(0, f32_dev(dY.reshape(T, H)), dX, sv, dA, dB)
        for p in masters:
            hb.adamw_step(masters[p][0], mom[p][0], mom[p][1], dA[p], case.A_dev[p], step=t, zero_grad=True, **kw)
            hb.adamw_step(masters[p][1], mom[p][2], mom[p][3], dB[p], case.B_dev[p], step=t, zero_grad=True, **kw)
        torch.cuda.synchronize()
        # ---- oracle: the same loop; the forward pass sees bf16-rounded adapters like the kernels do
        used = {p: (wl.bf16_round(a.astype(np.float32)).astype(np.float64), wl.bf16_round(b.astype(np.float32)).astype(np.float64))
                for p, (a, b) in o_lora.items()}
        Yo, saved = O.layer_forward(case.X_np, case.W_np, used, case.lora.scale, sh)
        lo, dYo = O.mse_loss(Yo, case.T_np)
        ora_loss.append(lo)
        _, grads = O.layer_backward(dYo, saved, case.W_np, used, case.lora.scale, sh)
        for p in o_lora:
            a, ma, va = adamw_step(o_lora[p][0], grads[p][0], o_mom[p][0], o_mom[p][1], t, lr=5e-3, b1=0.9, b2=0.99, eps=1e-8)
            b, mb, vb = adamw_step(o_lora[p][1], grads[p][1], o_mom[p][2], o_mom[p][3], t, lr=5e-3, b1=0.9, b2=0.99, eps=1e-8)
            o_lora[p] = (a, b)
            o_mom[p] = [ma, va, mb, vb]
    print("loss GPU   ", ["%.6f" % x for x in gpu_loss])
    print("loss oracle", ["%.6f" % x for x in ora_loss])
    assert gpu_loss[-1] < gpu_loss[0] and ora_loss[-1] < ora_loss[0]
    assert np.allclose(gpu_loss, ora_loss, rtol=5e-3)
    for p in o_lora:
        for got, want in ((masters[p][0], o_lora[p][0]), (masters[p][1], o_lora[p][1])):
            g = got.cpu().numpy().astype(np.float64)
            assert np.linalg.norm(g - want) <= 2e-2 * np.linalg.norm(want), p
