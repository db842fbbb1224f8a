"""Pins of the AdamW oracle (CPU only): closed forms and an independent library implementation."""
import numpy as np
import torch

from oracle.optim_oracle import adamw_step


def test_first_step_is_lr_times_normalised_gradient():
    g = np.array([0.5, -2.0, 1e-3, 0.0])
    p0 = np.array([1.0, 1.0, 1.0, 1.0])
    p, m, v = adamw_step(p0, g, np.zeros(4), np.zeros(4), 1, lr=0.01, eps=1e-8, wd=0.0)
    want = p0 - 0.01 * g / (np.abs(g) + 1e-8)        # bias corrections cancel at t = 1
    assert np.allclose(p, want, rtol=0, atol=1e-15)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_zero_gradient_only_decays():
    p0 = np.array([2.0, -4.0])
    p, m, v = adamw_step(p0, np.zeros(2), np.zeros(2), np.zeros(2), 1, lr=0.1, wd=0.05)
    assert np.allclose(p, p0 * (1 - 0.1 * 0.05)) and not m.any() and not v.any()


def test_constant_gradient_walks_at_constant_speed():
    g = np.array([3.0, -0.25])
    p, m, v = np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 21):
        p, m, v = adamw_step(p, g, m, v, t, lr=1e-2, eps=1e-8, wd=0.0)
    # m_hat = g and v_hat = g^2 at every step
    assert np.allclose(p, -20 * 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-12)


def test_matches_torch_adamw_over_many_steps():
    rng = np.random.default_rng(3)
    p0 = rng.standard_normal(257)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=3e-3, betas=(0.9, 0.95), eps=1e-6, weight_decay=0.1)
    p, m, v = p0.copy(), np.zeros(257), np.zeros(257)
    for t in range(1, 31):
        g = rng.standard_normal(257) * (1.0 + 0.1 * t)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = adamw_step(p, g, m, v, t, lr=3e-3, b1=0.9, b2=0.95, eps=1e-6, wd=0.1)
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-10, atol=1e-12), t


def test_grad_scale_is_applied_before_the_moments():
    g = np.array([4.0, -8.0])
    a = adamw_step(np.ones(2), g, np.zeros(2), np.zeros(2), 1, grad_scale=0.25)
    b = adamw_step(np.ones(2), g * 0.25, np.zeros(2), np.zeros(2), 1)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
