"""Pins for the oracle's temperature-softmax KL distillation loss."""
import math

import numpy as np
import pytest

from oracle.kd import kd_loss_forward_backward as kd
from conftest import fd_grad


def _make(rng, n=5, v=11, ht=6, hs=4):
    return (rng.standard_normal((n, ht)), rng.standard_normal((n, hs)),
            rng.standard_normal((v, ht)), rng.standard_normal((v, hs)))


def test_brute_force_tiny(rng):
    h_t, h_s, w_t, w_s = _make(rng, 3, 5, 4, 3)
    T, sc = 1.7, 0.25
    out = kd(h_t, h_s, w_t, w_s, T, sc)
    tot = 0.0
    for t in range(3):
        zt = [sum(h_t[t, i] * w_t[v, i] for i in range(4)) / T for v in range(5)]
        zs = [sum(h_s[t, i] * w_s[v, i] for i in range(3)) / T for v in range(5)]
        p = [math.exp(z) / sum(math.exp(x) for x in zt) for z in zt]
        q = [math.exp(z) / sum(math.exp(x) for x in zs) for z in zs]
        kl = sum(p[v] * math.log(p[v] / q[v]) for v in range(5))
        assert out["kl_tok"][t] == pytest.approx(kl, rel=1e-12)
        tot += kl
        for i in range(3):
            ref = sum(sc / T * (q[v] - p[v]) * w_s[v, i] for v in range(5))
            assert out["d_h_s"][t, i] == pytest.approx(ref, rel=1e-10, abs=1e-14)
    assert out["loss"] == pytest.approx(sc * tot, rel=1e-12)


def test_nonnegative_and_zero_for_equal_or_shifted_logits(rng):
    h_t, h_s, w_t, w_s = _make(rng)
    assert np.all(kd(h_t, h_s, w_t, w_s, 2.0, 1.0)["kl_tok"] > 0)
    same = kd(h_s, h_s, w_s, w_s, 2.0, 1.0)
    assert np.allclose(same["kl_tok"], 0, atol=1e-14) and np.allclose(same["d_w_s"], 0, atol=1e-14)
    # teacher logits = student logits + 3.5 for every vocab entry: still the same distribution
    h_t2 = np.concatenate([h_s, np.ones((h_s.shape[0], 1))], axis=1)
    w_t2 = np.concatenate([w_s, 3.5 * np.ones((w_s.shape[0], 1))], axis=1)
    sh = kd(h_t2, h_s, w_t2, w_s, 2.0, 1.0)
    assert np.allclose(sh["kl_tok"], 0, atol=1e-13) and np.allclose(sh["d_h_s"], 0, atol=1e-13)


def test_uniform_student_closed_form(rng):
    h_t, h_s, w_t, w_s = _make(rng)
    out = kd(h_t, h_s, w_t, 0 * w_s, 1.3, 1.0)
    z = h_t @ w_t.T / 1.3
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    ent = -np.sum(p * np.log(p), axis=1)
    assert np.allclose(out["kl_tok"], math.log(11) - ent, atol=1e-13)           # ln V - H(p)


def test_temperature_limits_and_scaling(rng):
    h_t, h_s, w_t, w_s = _make(rng)
    assert np.all(kd(h_t, h_s, w_t, w_s, 1e6, 1.0)["kl_tok"] < 1e-9)            # T -> inf: both uniform
    a = kd(h_t, h_s, w_t, w_s, 2.5, 1.0)
    b = kd(h_t, h_s, w_t / 2.5, w_s / 2.5, 1.0, 1.0)
    assert np.allclose(a["kl_tok"], b["kl_tok"], atol=1e-14)
    assert np.allclose(a["d_h_s"], b["d_h_s"], atol=1e-14)                      # dz/T * Ws == dz * (Ws/T)


def test_logit_gradient_sums_to_zero(rng):
    # with Ws = I the hidden gradient IS the logit gradient; softmax differences sum to zero per token
    h_t, _, w_t, _ = _make(rng, v=4, hs=4)
    h_s = rng.standard_normal((5, 4))
    out = kd(h_t, h_s, w_t, np.eye(4), 1.5, 0.2)
    assert np.allclose(out["d_h_s"].sum(axis=1), 0, atol=1e-15)
    assert np.any(np.abs(out["d_h_s"]) > 1e-3)


def test_finite_difference_gradients(rng):
    h_t, h_s, w_t, w_s = _make(rng)
    T, sc = 2.0, 1.0 / 5
    f = lambda: kd(h_t, h_s, w_t, w_s, T, sc, need_grad=False)["loss"]
    out = kd(h_t, h_s, w_t, w_s, T, sc)
    for idx in [(0, 0), (2, 3), (4, 1)]:
        assert out["d_h_s"][idx] == pytest.approx(fd_grad(f, h_s, idx), rel=1e-6, abs=1e-10)
    for idx in [(0, 0), (10, 3), (5, 2)]:
        assert out["d_w_s"][idx] == pytest.approx(fd_grad(f, w_s, idx), rel=1e-6, abs=1e-10)


def test_token_block_invariance(rng):
    h_t, h_s, w_t, w_s = _make(rng, n=13)
    a = kd(h_t, h_s, w_t, w_s, 2.0, 1 / 13, token_block=13)
    b = kd(h_t, h_s, w_t, w_s, 2.0, 1 / 13, token_block=4)
    assert np.allclose(a["kl_tok"], b["kl_tok"], atol=1e-15) and a["loss"] == pytest.approx(b["loss"], rel=1e-14)
    assert np.allclose(a["d_w_s"], b["d_w_s"], atol=1e-15) and np.allclose(a["d_h_s"], b["d_h_s"], atol=1e-16)
