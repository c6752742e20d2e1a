"""Pins of the AdamW oracle: closed forms, invariants and torch's own optimizer as a library special case."""
import numpy as np
import pytest
import torch

from oracle.optimizer import adamw_step


def test_first_step_is_a_signed_step():
    # t = 1: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps): lr * sign(g) for |g| >> eps
    g = np.array([0.5, -2.0, 1e-3, -7.0])
    w, m, v, _ = adamw_step(np.zeros(4), np.zeros(4), np.zeros(4), g, 1, lr=0.1, eps=0.0)
    np.testing.assert_allclose(w, -0.1 * np.sign(g), rtol=1e-9)
    np.testing.assert_allclose(m, 0.1 * g)
    np.testing.assert_allclose(v, 0.05 * g * g)


def test_zero_gradient_only_decays():
    w0 = np.array([1.0, -3.0])
    w, m, v, _ = adamw_step(w0, np.zeros(2), np.zeros(2), np.zeros(2), 5, lr=0.01, weight_decay=0.1)
    np.testing.assert_allclose(w, w0 * (1 - 0.001))                     # decoupled decay: no gradient term
    assert not m.any() and not v.any()


def test_constant_gradient_closed_form():
    # constant g: m_hat = g and v_hat = g^2 at every step, so without decay w_t = w_0 - t lr sign(g)
    g, w, m, v = np.array([0.3, -0.3]), np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 8):
        w, m, v, _ = adamw_step(w, m, v, g, t, lr=0.01, eps=0.0)
    np.testing.assert_allclose(w, -7 * 0.01 * np.sign(g), rtol=1e-12)


def test_grad_scale_and_rounding_hooks():
    g = np.array([1.0, 2.0, -4.0])
    a = adamw_step(np.ones(3), np.zeros(3), np.zeros(3), g, 1, lr=0.1, grad_scale=0.5)
    b = adamw_step(np.ones(3), np.zeros(3), np.zeros(3), 0.5 * g, 1, lr=0.1)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y)
    from oracle import round_bf16
    *_, wm = adamw_step(np.ones(3), np.zeros(3), np.zeros(3), g, 1, lr=0.003, rnd=round_bf16)
    assert np.all(wm == round_bf16(wm)) and np.any(wm != a[0])


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_against_torch_adamw(wd):
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal(257)
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    w, m, v = w0.copy(), np.zeros(257), np.zeros(257)
    for t in range(1, 6):
        g = rng.standard_normal(257) * (1.0 + t)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v, _ = adamw_step(w, m, v, g, t, lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=wd)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-10, atol=1e-12)
