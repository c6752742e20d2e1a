"""Pins for the oracle's layer building blocks: closed forms, brute force, invariants,
finite differences.  None of these retype the oracle's own vectorised formula."""
import math

import numpy as np
import pytest
import torch

from oracle import ops, round_bf16
from conftest import fd_grad


def test_round_bf16_matches_torch_and_ties_to_even(rng):
    x = rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))
    ref = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_bf16(x), ref)
    assert round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0                    # tie -> even (down)
    assert round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6    # tie -> even (up)
    assert round_bf16(np.array([-0.15625]))[0] == -0.15625                       # representable


def test_linear_against_triple_loop(rng):
    x, w, b = rng.standard_normal((5, 7)), rng.standard_normal((3, 7)), rng.standard_normal(3)
    dy = rng.standard_normal((5, 3))
    y = ops.linear_fwd(x, w, b)
    dx, dw, db = ops.linear_bwd(dy, x, w, True)
    for t in range(5):
        for o in range(3):
            assert y[t, o] == pytest.approx(sum(x[t, i] * w[o, i] for i in range(7)) + b[o], rel=1e-12)
    for t in range(5):
        for i in range(7):
            assert dx[t, i] == pytest.approx(sum(dy[t, o] * w[o, i] for o in range(3)), rel=1e-12)
    for o in range(3):
        assert db[o] == pytest.approx(sum(dy[t, o] for t in range(5)), rel=1e-12)
        for i in range(7):
            assert dw[o, i] == pytest.approx(sum(dy[t, o] * x[t, i] for t in range(5)), rel=1e-12)


def test_rmsnorm_properties_and_brute_force(rng):
    x = rng.standard_normal((6, 16)) * 3
    g = 1 + 0.1 * rng.standard_normal(16)
    y, r = ops.rmsnorm_fwd(x, np.ones(16), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, atol=1e-12)       # unit rms
    y2, _ = ops.rmsnorm_fwd(7.5 * x, np.ones(16), 0.0)
    assert np.allclose(y, y2, atol=1e-12)                                      # scale invariant
    eps = 1e-3
    yg, rg = ops.rmsnorm_fwd(x, g, eps)
    for t in range(6):
        ms = sum(v * v for v in x[t]) / 16
        for j in range(16):
            assert yg[t, j] == pytest.approx(x[t, j] / math.sqrt(ms + eps) * g[j], rel=1e-12)
        assert rg[t] == pytest.approx(1 / math.sqrt(ms + eps), rel=1e-12)


def test_rmsnorm_backward_finite_difference(rng):
    x, g, c = rng.standard_normal((4, 12)), 1 + 0.2 * rng.standard_normal(12), rng.standard_normal((4, 12))
    eps = 1e-5
    f = lambda: float(np.sum(c * ops.rmsnorm_fwd(x, g, eps)[0]))
    _, r = ops.rmsnorm_fwd(x, g, eps)
    dx, dg = ops.rmsnorm_bwd(c, x, r, g)
    for idx in [(0, 0), (1, 5), (3, 11), (2, 7)]:
        assert dx[idx] == pytest.approx(fd_grad(f, x, idx), rel=1e-6, abs=1e-9)
    for j in [0, 4, 11]:
        assert dg[j] == pytest.approx(fd_grad(f, g, j), rel=1e-6, abs=1e-9)
    _, r0 = ops.rmsnorm_fwd(x, g, 0.0)
    dx0, _ = ops.rmsnorm_bwd(c, x, r0, g)
    assert np.allclose(np.sum(dx0 * x, axis=1), 0.0, atol=1e-12)              # scale invariance => dx . x = 0


def test_layernorm_properties_and_backward(rng):
    x = rng.standard_normal((5, 10)) * 2 + 3
    g, b, c = 1 + 0.2 * rng.standard_normal(10), rng.standard_normal(10), rng.standard_normal((5, 10))
    y, mu, r = ops.layernorm_fwd(x, np.ones(10), np.zeros(10), 0.0)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12) and np.allclose(y.var(axis=1), 1, atol=1e-12)
    assert np.allclose(mu, x.mean(axis=1))
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (10,), torch.tensor(g), torch.tensor(b), 1e-6).numpy()
    assert np.allclose(ops.layernorm_fwd(x, g, b, 1e-6)[0], ref, atol=1e-12)   # library routine
    eps = 1e-5
    f = lambda: float(np.sum(c * ops.layernorm_fwd(x, g, b, eps)[0]))
    _, mu, r = ops.layernorm_fwd(x, g, b, eps)
    dx, dg, db = ops.layernorm_bwd(c, x, mu, r, g)
    for idx in [(0, 0), (4, 9), (2, 3)]:
        assert dx[idx] == pytest.approx(fd_grad(f, x, idx), rel=1e-6, abs=1e-9)
    for j in [0, 9]:
        assert dg[j] == pytest.approx(fd_grad(f, g, j), rel=1e-6, abs=1e-9)
        assert db[j] == pytest.approx(fd_grad(f, b, j), rel=1e-6, abs=1e-9)
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-12)                          # shift invariance


def test_rope_closed_forms(rng):
    # hd = 2: a single pair rotated by pos * base^0 = pos radians
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -1.0]]])
    pos = np.array([1, 2, 0])
    y = ops.rope_apply(x, pos, 1e4)
    assert y[0, 0] == pytest.approx([math.cos(1), math.sin(1)])
    assert y[1, 0] == pytest.approx([-math.sin(2), math.cos(2)])
    assert np.array_equal(y[2], x[2])                                           # pos 0 is the identity
    # hd = 4: pair (1, 3) uses theta = base^(-2/4) = 0.01 for base 1e4; pairs are (i, i + hd/2)
    x4 = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    y4 = ops.rope_apply(x4, np.array([3]), 1e4)
    assert y4[0, 0] == pytest.approx([0.0, math.cos(0.03), 0.0, math.sin(0.03)])


def test_rope_invariants(rng):
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    for hd_pos in [(5, 2), (105, 102), (40, 37)]:
        a = ops.rope_apply(q, np.array([hd_pos[0]]), 1e4)
        b = ops.rope_apply(k, np.array([hd_pos[1]]), 1e4)
        if hd_pos == (5, 2):
            ref = float(np.sum(a * b))
        assert float(np.sum(a * b)) == pytest.approx(ref, rel=1e-9)            # depends on m - n only
        assert np.linalg.norm(a) == pytest.approx(np.linalg.norm(q))           # norm preserving
    x, y = rng.standard_normal((7, 3, 8)), rng.standard_normal((7, 3, 8))
    pos = np.arange(7)
    lhs = np.sum(ops.rope_apply(x, pos, 100.0) * y)
    rhs = np.sum(x * ops.rope_apply(y, pos, 100.0, inverse=True))
    assert lhs == pytest.approx(rhs, rel=1e-12)                                 # backward is the transpose
    assert np.array_equal(ops.positions_from_cu([0, 3, 3, 5]), [0, 1, 2, 0, 1])


def test_swiglu_values_and_backward(rng):
    gu = np.array([[0.0, 1.0, 30.0, 5.0, 2.0, 3.0]])
    a = ops.swiglu_fwd(gu)
    assert a[0, 0] == 0.0
    assert a[0, 1] == pytest.approx(0.7310585786300049 * 2.0)                   # silu(1) * up
    assert a[0, 2] == pytest.approx(30.0 * 3.0, rel=1e-12)                      # silu(x) -> x
    gu = rng.standard_normal((3, 8))
    c = rng.standard_normal((3, 4))
    f = lambda: float(np.sum(c * ops.swiglu_fwd(gu)))
    d = ops.swiglu_bwd(c, gu)
    for idx in [(0, 0), (1, 3), (2, 4), (0, 7)]:
        assert d[idx] == pytest.approx(fd_grad(f, gu, idx), rel=1e-6, abs=1e-9)


def test_gelu_values_and_backward(rng):
    x = np.array([0.0, 1.0, -1.0, 12.0, -12.0])
    y = ops.gelu_fwd(x)
    assert y[0] == 0.0
    assert y[1] == pytest.approx(0.8413447460685429)                            # Phi(1)
    assert y[2] == pytest.approx(-0.15865525393145707)                          # -Phi(-1)
    assert y[3] == pytest.approx(12.0) and abs(y[4]) < 1e-30
    x = rng.standard_normal((3, 5))
    c = rng.standard_normal((3, 5))
    f = lambda: float(np.sum(c * ops.gelu_fwd(x)))
    d = ops.gelu_bwd(c, x)
    for idx in [(0, 0), (1, 3), (2, 4)]:
        assert d[idx] == pytest.approx(fd_grad(f, x, idx), rel=1e-6, abs=1e-9)
    ref = torch.nn.functional.gelu(torch.tensor(x)).numpy()
    assert np.allclose(ops.gelu_fwd(x), ref, atol=1e-14)


def test_embedding_gather_and_scatter_add(rng):
    e = rng.standard_normal((6, 3))
    ids = np.array([4, 0, 4, 5])
    assert np.array_equal(ops.embedding_fwd(ids, e), e[[4, 0, 4, 5]])
    dx = rng.standard_normal((4, 3))
    de = ops.embedding_bwd(ids, dx, 6)
    assert np.allclose(de[4], dx[0] + dx[2]) and np.allclose(de[0], dx[1]) and np.allclose(de[5], dx[3])
    assert np.all(de[[1, 2, 3]] == 0)
