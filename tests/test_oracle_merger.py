"""Pins of the vision -> language hand-off oracle: index bookkeeping against a loop written out by hand, gradients
against central differences, and the special cases that reduce to a plain linear map."""
import numpy as np

from oracle.merger import merger_backward, merger_forward
from oracle.ops import gelu_fwd


def setup(seed=0, g=5, merge=4, dv=6, dh=10, dl=7, n_llm=12):
    r = np.random.default_rng(seed)
    h = r.standard_normal((g * merge, dv))
    w1, b1 = r.standard_normal((dh, merge * dv)) * 0.3, r.standard_normal(dh) * 0.1
    w2, b2 = r.standard_normal((dl, dh)) * 0.3, r.standard_normal(dl) * 0.1
    pos = r.permutation(n_llm)[:g]
    x = r.standard_normal((n_llm, dl))
    return h, w1, b1, w2, b2, pos, x


def test_forward_against_a_hand_written_loop():
    h, w1, b1, w2, b2, pos, x = setup()
    out, _ = merger_forward(h, w1, b1, w2, b2, pos, x)
    ref = x.copy()
    for gi in range(len(pos)):                                   # group gi = visual tokens 4 gi .. 4 gi + 3, in order
        cat = np.concatenate([h[4 * gi + j] for j in range(4)])
        a1 = w1 @ cat + b1
        ref[pos[gi]] = w2 @ gelu_fwd(a1) + b2
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    text = np.setdiff1d(np.arange(x.shape[0]), pos)
    assert np.array_equal(out[text], x[text])                    # text rows are left alone


def test_gradients_against_central_differences():
    h, w1, b1, w2, b2, pos, x = setup(1)
    r = np.random.default_rng(9)
    d_x = r.standard_normal(x.shape)

    def loss(h_, w1_, b1_, w2_, b2_):
        return float(np.sum(merger_forward(h_, w1_, b1_, w2_, b2_, pos, x)[0] * d_x))
    _, cache = merger_forward(h, w1, b1, w2, b2, pos, x)
    d_h, gw = merger_backward(d_x, cache, w1, w2, pos)
    args = [h, w1, b1, w2, b2]
    for k, (name, got) in enumerate([("h", d_h), ("w1", gw["w1"]), ("b1", gw["b1"]), ("w2", gw["w2"]), ("b2", gw["b2"])]):
        for _ in range(6):
            idx = tuple(r.integers(0, s) for s in args[k].shape)
            e = np.zeros_like(args[k]); e[idx] = 1e-6
            plus = [a + e if j == k else a for j, a in enumerate(args)]
            minus = [a - e if j == k else a for j, a in enumerate(args)]
            fd = (loss(*plus) - loss(*minus)) / 2e-6
            assert abs(fd - got[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, got[idx])


def test_text_positions_get_no_gradient_path():
    h, w1, b1, w2, b2, pos, x = setup(2)
    _, cache = merger_forward(h, w1, b1, w2, b2, pos, x)
    d_x = np.zeros_like(x)
    text = np.setdiff1d(np.arange(x.shape[0]), pos)
    d_x[text] = 1.0                                              # gradient only on text rows
    d_h, gw = merger_backward(d_x, cache, w1, w2, pos)
    assert not d_h.any() and not gw["w1"].any() and not gw["b2"].any()


def test_merge_one_is_a_two_layer_mlp_on_each_token():
    h, w1, b1, w2, b2, pos, x = setup(3, g=6, merge=1, dv=5)
    out, _ = merger_forward(h, w1, b1, w2, b2, pos, x, merge=1)
    np.testing.assert_allclose(out[pos], gelu_fwd(h @ w1.T + b1) @ w2.T + b2, rtol=1e-12)
