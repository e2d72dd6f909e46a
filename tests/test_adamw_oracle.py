"""Pins for the AdamW oracle: the library optimizer in float64 and a closed form for the first step."""
import numpy as np
import torch

from oracle.adamw_oracle import Hyper, adamw_step


def test_matches_torch_adamw_float64_over_several_steps():
    rng = np.random.default_rng(0)
    theta0 = rng.standard_normal((7, 5))
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.05)
    th, m, v = theta0.copy(), np.zeros_like(theta0), np.zeros_like(theta0)
    for t in range(1, 6):
        g = rng.standard_normal(theta0.shape)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = adamw_step(th, g, m, v, Hyper(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.05, step=t))
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_first_step_closed_form():
    # t = 1, zero state: mh = g, vh = g^2, so theta1 = theta0 (1 - lr wd) - lr g / (|g| + eps)
    th0 = np.array([1.0, -2.0, 0.5]); g = np.array([0.25, -4.0, 1e-3])
    hp = Hyper(lr=0.1, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1)
    th1, m1, v1 = adamw_step(th0, g, np.zeros(3), np.zeros(3), hp)
    np.testing.assert_allclose(th1, th0 * (1 - 0.1 * 0.01) - 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-15)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_zero_gradient_only_decays():
    th0 = np.array([2.0, -3.0])
    th1, m1, v1 = adamw_step(th0, np.zeros(2), np.zeros(2), np.zeros(2), Hyper(lr=0.5, weight_decay=0.1, step=3))
    np.testing.assert_allclose(th1, th0 * (1 - 0.05), rtol=1e-15)
    assert np.all(m1 == 0) and np.all(v1 == 0)
