"""Pins for the oracle's dense variable-length attention."""
import math

import numpy as np
import pytest

from oracle.attention import attention_bwd, attention_fwd
from conftest import fd_grad


def _brute(q, k, v, cu, causal):
    n, nq, hd = q.shape
    grp = nq // k.shape[1]
    o = np.zeros_like(q)
    for b in range(len(cu) - 1):
        for i in range(cu[b], cu[b + 1]):
            for h in range(nq):
                last = i if causal else cu[b + 1] - 1
                s = [sum(q[i, h, d] * k[j, h // grp, d] for d in range(hd)) / math.sqrt(hd)
                     for j in range(cu[b], last + 1)]
                m = max(s)
                e = [math.exp(x - m) for x in s]
                z = sum(e)
                for d in range(hd):
                    o[i, h, d] = sum(e[jj] / z * v[cu[b] + jj, h // grp, d] for jj in range(len(s)))
    return o


@pytest.mark.parametrize("causal", [True, False])
def test_brute_force_tiny(rng, causal):
    cu = [0, 3, 4, 9]
    q, k, v = rng.standard_normal((9, 4, 4)), rng.standard_normal((9, 2, 4)), rng.standard_normal((9, 2, 4))
    assert np.allclose(attention_fwd(q, k, v, cu, causal), _brute(q, k, v, cu, causal), atol=1e-13)


def test_log_sum_exp_against_loops(rng):
    cu = [0, 3, 7]
    q, k, v = rng.standard_normal((7, 2, 4)), rng.standard_normal((7, 1, 4)), rng.standard_normal((7, 1, 4))
    _, lse = attention_fwd(q, k, v, cu, True, return_lse=True)
    for b in range(2):
        for i in range(cu[b], cu[b + 1]):
            for h in range(2):
                tot = sum(math.exp(sum(q[i, h, d] * k[j, 0, d] for d in range(4)) / 2.0) for j in range(cu[b], i + 1))
                assert lse[h, i] == pytest.approx(math.log(tot), rel=1e-12)


def test_length_one_and_equal_keys(rng):
    q, k, v = rng.standard_normal((1, 2, 8)), rng.standard_normal((1, 2, 8)), rng.standard_normal((1, 2, 8))
    assert np.allclose(attention_fwd(q, k, v, [0, 1], True), v)
    L = 6
    q, v = rng.standard_normal((L, 1, 8)), rng.standard_normal((L, 1, 8))
    k = np.tile(rng.standard_normal((1, 1, 8)), (L, 1, 1))
    oc = attention_fwd(q, k, v, [0, L], True)
    ob = attention_fwd(q, k, v, [0, L], False)
    for i in range(L):
        assert np.allclose(oc[i, 0], v[:i + 1, 0].mean(axis=0))                 # running mean
        assert np.allclose(ob[i, 0], v[:, 0].mean(axis=0))


def test_causality_is_bit_exact(rng):
    q, k, v = rng.standard_normal((10, 2, 8)), rng.standard_normal((10, 2, 8)), rng.standard_normal((10, 2, 8))
    o1 = attention_fwd(q, k, v, [0, 10], True)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[6:] += 1.0; k2[6:] -= 2.0; v2[6:] *= 3.0
    o2 = attention_fwd(q2, k2, v2, [0, 10], True)
    assert np.array_equal(o1[:6], o2[:6]) and not np.allclose(o1[6:], o2[6:])
    ob1 = attention_fwd(q, k, v, [0, 10], False)
    ob2 = attention_fwd(q, k2, v2, [0, 10], False)
    assert not np.allclose(ob1[:6], ob2[:6])                                    # encoder does look ahead


@pytest.mark.parametrize("causal", [True, False])
def test_packed_equals_separate_and_no_cross_talk(rng, causal):
    lens = [5, 1, 7]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v = rng.standard_normal((13, 4, 8)), rng.standard_normal((13, 2, 8)), rng.standard_normal((13, 2, 8))
    o = attention_fwd(q, k, v, cu, causal)
    for b in range(3):
        s = slice(cu[b], cu[b + 1])
        assert np.array_equal(o[s], attention_fwd(q[s], k[s], v[s], [0, lens[b]], causal))
    # zero-length entries in cu_seqlens are legal and change nothing
    assert np.array_equal(o, attention_fwd(q, k, v, [0, 5, 5, 6, 13, 13], causal))


def test_gqa_equals_mha_with_replicated_kv(rng):
    q, k, v = rng.standard_normal((7, 6, 4)), rng.standard_normal((7, 2, 4)), rng.standard_normal((7, 2, 4))
    kr, vr = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    assert np.allclose(attention_fwd(q, k, v, [0, 7], True), attention_fwd(q, kr, vr, [0, 7], True), atol=1e-15)
    do = rng.standard_normal((7, 6, 4))
    dq, dk, dv = attention_bwd(do, q, k, v, [0, 7], True)
    dq2, dk2, dv2 = attention_bwd(do, q, kr, vr, [0, 7], True)
    assert np.allclose(dq, dq2)
    assert np.allclose(dk, dk2.reshape(7, 2, 3, 4).sum(axis=2))                 # group sum
    assert np.allclose(dv, dv2.reshape(7, 2, 3, 4).sum(axis=2))


def test_encoder_is_permutation_equivariant(rng):
    q, k, v = rng.standard_normal((8, 2, 4)), rng.standard_normal((8, 2, 4)), rng.standard_normal((8, 2, 4))
    perm = rng.permutation(8)
    o = attention_fwd(q, k, v, [0, 8], False)
    op = attention_fwd(q[perm], k[perm], v[perm], [0, 8], False)
    assert np.allclose(o[perm], op, atol=1e-14)


def test_sharp_scores_stay_finite(rng):
    q, k, v = 60 * rng.standard_normal((12, 1, 8)), 60 * rng.standard_normal((12, 1, 8)), rng.standard_normal((12, 1, 8))
    o = attention_fwd(q, k, v, [0, 12], False)
    assert np.all(np.isfinite(o))
    # near one-hot rows: each output is (almost) one of the value rows
    d = np.abs(o[:, 0, None, :] - v[None, :, 0, :]).max(axis=2).min(axis=1)
    assert np.all(d < 1e-6)


@pytest.mark.parametrize("causal", [True, False])
def test_backward_finite_difference(rng, causal):
    cu = [0, 4, 9]
    q, k, v = rng.standard_normal((9, 4, 4)), rng.standard_normal((9, 2, 4)), rng.standard_normal((9, 2, 4))
    c = rng.standard_normal((9, 4, 4))
    f = lambda: float(np.sum(c * attention_fwd(q, k, v, cu, causal)))
    dq, dk, dv = attention_bwd(c, q, k, v, cu, causal)
    # the stored-output form of the row term (rowsum(dO * O)) is the same gradient
    for a, b in zip((dq, dk, dv), attention_bwd(c, q, k, v, cu, causal, o=attention_fwd(q, k, v, cu, causal))):
        assert np.allclose(a, b, atol=1e-13)
    for idx in [(0, 0, 0), (3, 1, 2), (5, 3, 1), (8, 2, 3)]:
        assert dq[idx] == pytest.approx(fd_grad(f, q, idx), rel=1e-6, abs=1e-9)
    for idx in [(0, 0, 0), (3, 1, 2), (5, 0, 1), (8, 1, 3)]:
        assert dk[idx] == pytest.approx(fd_grad(f, k, idx), rel=1e-6, abs=1e-9)
        assert dv[idx] == pytest.approx(fd_grad(f, v, idx), rel=1e-6, abs=1e-9)


@pytest.mark.parametrize("causal", [True, False])
def test_operand_rounding_hook_sees_p_and_ds_only(rng, causal):
    """rnd_p is applied to P (for dV) and to dS = P * (dP - delta) (for dQ, dK), and to nothing else."""
    from oracle import round_bf16
    L, hd = 5, 4
    q, k, v, do = (rng.standard_normal((L, 1, hd)) for _ in range(4))
    # P, dP, delta by loops
    P = np.zeros((L, L))
    for i in range(L):
        js = range(i + 1) if causal else range(L)
        e = {j: math.exp(sum(q[i, 0, d] * k[j, 0, d] for d in range(hd)) / math.sqrt(hd)) for j in js}
        z = sum(e.values())
        for j in js:
            P[i, j] = e[j] / z
    dP = np.array([[sum(do[i, 0, d] * v[j, 0, d] for d in range(hd)) for j in range(L)] for i in range(L)])
    delta = np.array([sum(P[i, j] * dP[i, j] for j in range(L)) for i in range(L)])
    dS = P * (dP - delta[:, None])
    seen = []
    def hook(x):
        seen.append(np.array(x))
        return 2.0 * x                      # not a rounding: makes every use of the hook's output visible
    dq, dk, dv = attention_bwd(do, q, k, v, [0, L], causal, rnd_p=hook)
    assert len(seen) == 2 and np.allclose(seen[0], P, atol=1e-14) and np.allclose(seen[1], dS, atol=1e-14)
    dq0, dk0, dv0 = attention_bwd(do, q, k, v, [0, L], causal)
    # each gradient is linear in exactly one hooked matrix (dP and delta do not pass through the hook: no factor 4)
    assert np.allclose(dq, 2 * dq0) and np.allclose(dk, 2 * dk0) and np.allclose(dv, 2 * dv0)
    # with the bf16 rounding the gradients stay within the rounding bound |x - rnd(x)| <= 2^-8 |x| of each operand element
    dqr, dkr, dvr = attention_bwd(do, q, k, v, [0, L], causal, rnd_p=round_bf16)
    u = 2.0 ** -8                            # half an ulp of an 8-bit significand
    assert np.all(np.abs(dvr - dv0)[:, 0] <= u * (P.T @ np.abs(do[:, 0])) + 1e-15)
    assert np.all(np.abs(dqr - dq0)[:, 0] <= u * (np.abs(dS) @ np.abs(k[:, 0])) / math.sqrt(hd) + 1e-15)
    assert np.all(np.abs(dkr - dk0)[:, 0] <= u * (np.abs(dS).T @ np.abs(q[:, 0])) / math.sqrt(hd) + 1e-15)
    assert not np.array_equal(dqr, dq0)
