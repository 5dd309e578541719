"""Pins for the optimizer-step oracle (Table 2 "OS"; AdamW is this build's reading)."""
import numpy as np
import torch

from oracle import optimizer_oracle as OO


def test_matches_torch_adamw_over_several_steps():
    rng = np.random.default_rng(0)
    n, lr, b1, b2, eps, wd = 257, 3e-3, 0.85, 0.97, 1e-6, 0.02
    theta0 = rng.normal(size=n)
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    th, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = rng.normal(size=n) * (1.0 + t)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = OO.adamw_step(th, g, m, v, t, lr, b1, b2, eps, wd)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12)


def test_first_step_closed_form_and_gradient_scale():
    g = np.array([2.0, -0.5, 0.0, 1e-3])
    th, m, v = OO.adamw_step(np.ones(4), g, np.zeros(4), np.zeros(4), 1, lr=0.1, eps=1e-8)
    np.testing.assert_allclose(th, 1.0 - 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-14)   # m_hat = g, v_hat = g^2
    np.testing.assert_allclose(m, 0.1 * g)
    np.testing.assert_allclose(v, 1e-3 * g * g)
    a = OO.adamw_step(np.ones(4), g, np.zeros(4), np.zeros(4), 1, lr=0.1, grad_scale=0.25)
    b = OO.adamw_step(np.ones(4), 0.25 * g, np.zeros(4), np.zeros(4), 1, lr=0.1)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-15)


def test_zero_gradient_leaves_only_the_decoupled_decay():
    th0 = np.array([1.5, -2.0, 0.25])
    th, m, v = OO.adamw_step(th0, np.zeros(3), np.zeros(3), np.zeros(3), 3, lr=0.01, weight_decay=0.1)
    np.testing.assert_allclose(th, th0 * (1 - 0.01 * 0.1), rtol=1e-15)
    assert not m.any() and not v.any()
    # the decay does not pass through the moments: with a gradient, changing weight_decay changes theta only
    g = np.array([0.3, -0.1, 0.2])
    a = OO.adamw_step(th0, g, np.zeros(3), np.zeros(3), 1, lr=0.01, weight_decay=0.0)
    b = OO.adamw_step(th0, g, np.zeros(3), np.zeros(3), 1, lr=0.01, weight_decay=0.5)
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(a[2], b[2])
    np.testing.assert_allclose(a[0] - b[0], 0.01 * 0.5 * th0, rtol=1e-12)


def test_constant_gradient_keeps_the_corrected_moments_at_g_and_g_squared():
    g = np.array([0.7, -1.3])
    th, m, v = np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 30):
        th, m, v = OO.adamw_step(th, g, m, v, t, lr=0.05, eps=0.0)
        np.testing.assert_allclose(m / (1 - 0.9 ** t), g, rtol=1e-12)
        np.testing.assert_allclose(v / (1 - 0.999 ** t), g * g, rtol=1e-12)
        np.testing.assert_allclose(th, -0.05 * t * np.sign(g), rtol=1e-10)   # each step moves by lr sign(g)
