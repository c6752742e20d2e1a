"""Pins for the oracle's section forward / backward (whole layer stacks, pure fp64)."""
import numpy as np
import pytest

from oracle import round_bf16
from oracle.section import SectionSpec, section_backward, section_forward
from oracle.step import distill_step
from conftest import fd_grad


def make_weights(rng, spec, scale=0.3):
    d, f, enc = spec.d_model, spec.d_ffn, spec.arch == "encoder"
    dqkv = (spec.n_q_heads + 2 * spec.n_kv_heads) * spec.head_dim
    dup = f if enc else 2 * f
    m = lambda *s: scale * rng.standard_normal(s)
    g = lambda: 1 + 0.1 * rng.standard_normal(d)
    w = {"layers": [], "final_norm_g": g()}
    if spec.vocab:
        w["embedding"] = rng.standard_normal((spec.vocab, d))
    if enc:
        w["final_norm_b"] = m(d)
    for _ in range(spec.n_layers):
        lw = dict(norm1_g=g(), w_qkv=m(dqkv, d), w_o=m(d, spec.n_q_heads * spec.head_dim),
                  norm2_g=g(), w_up=m(dup, d), w_down=m(d, f))
        if enc:
            lw.update(norm1_b=m(d), b_qkv=m(dqkv), b_o=m(d), norm2_b=m(d), b_up=m(dup), b_down=m(d))
        w["layers"].append(lw)
    return w


DEC = SectionSpec("decoder", 2, 8, 4, 2, 4, 6, vocab=0, norm_eps=1e-5, rope_base=100.0)
DEC_IDS = SectionSpec("decoder", 1, 8, 2, 2, 4, 6, vocab=7, norm_eps=1e-5, rope_base=100.0)
ENC = SectionSpec("encoder", 2, 8, 2, 2, 4, 10, vocab=0, norm_eps=1e-5)


@pytest.mark.parametrize("spec", [DEC, ENC], ids=["decoder", "encoder"])
def test_finite_difference_every_parameter_and_input(rng, spec):
    w = make_weights(rng, spec)
    cu = [0, 3, 3, 8]
    x = rng.standard_normal((8, spec.d_model))
    c = rng.standard_normal((8, spec.d_model))
    f = lambda: float(np.sum(c * section_forward(spec, w, cu, x)))
    _, cache = section_forward(spec, w, cu, x, keep=True)
    grads, dx = section_backward(spec, w, cu, cache, c)
    for idx in [(0, 0), (4, 5), (7, 7)]:
        assert dx[idx] == pytest.approx(fd_grad(f, x, idx), rel=2e-5, abs=1e-8)
    for name in w:
        if name == "layers":
            continue
        assert grads[name][3] == pytest.approx(fd_grad(f, w[name], 3), rel=2e-5, abs=1e-8)
    for li, lw in enumerate(w["layers"]):
        for name, arr in lw.items():
            for _ in range(2):
                idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
                assert grads["layers"][li][name][idx] == pytest.approx(
                    fd_grad(f, arr, idx), rel=2e-5, abs=1e-8), (li, name, idx)


def test_token_id_section_embedding_gradient(rng):
    w = make_weights(rng, DEC_IDS)
    cu, ids = [0, 4, 6], np.array([1, 5, 1, 0, 6, 1])
    c = rng.standard_normal((6, 8))
    f = lambda: float(np.sum(c * section_forward(DEC_IDS, w, cu, ids)))
    _, cache = section_forward(DEC_IDS, w, cu, ids, keep=True)
    grads, dx = section_backward(DEC_IDS, w, cu, cache, c)
    assert dx is None
    for idx in [(1, 0), (5, 3), (0, 7), (6, 2)]:
        assert grads["embedding"][idx] == pytest.approx(fd_grad(f, w["embedding"], idx), rel=2e-5, abs=1e-8)
    assert np.all(grads["embedding"][[2, 3, 4]] == 0)                           # ids never used


@pytest.mark.parametrize("spec", [DEC, ENC], ids=["decoder", "encoder"])
def test_packed_equals_separate_sequences(rng, spec):
    w = make_weights(rng, spec)
    lens = [5, 2, 6]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((13, spec.d_model))
    h = section_forward(spec, w, cu, x)
    for b in range(3):
        s = slice(cu[b], cu[b + 1])
        assert np.allclose(h[s], section_forward(spec, w, [0, lens[b]], x[s]), atol=1e-13)
    # a sample with no tokens for this section (skipped) changes nothing
    assert np.array_equal(h, section_forward(spec, w, [0, 5, 5, 7, 13], x))


def test_decoder_stack_is_causal_and_position_restarts(rng):
    w = make_weights(rng, DEC)
    x = rng.standard_normal((9, 8))
    h1 = section_forward(DEC, w, [0, 9], x)
    x2 = x.copy()
    x2[5:] += 1.0
    h2 = section_forward(DEC, w, [0, 9], x2)
    assert np.array_equal(h1[:5], h2[:5]) and not np.allclose(h1[5:], h2[5:])
    # the same 4 tokens placed second in a pack see positions 0..3 again
    xa = np.concatenate([rng.standard_normal((3, 8)), x[:4]])
    assert np.allclose(section_forward(DEC, w, [0, 3, 7], xa)[3:], section_forward(DEC, w, [0, 4], x[:4]), atol=1e-13)


def test_two_layers_compose(rng):
    w = make_weights(rng, DEC)
    x = rng.standard_normal((6, 8))
    one = SectionSpec(**{**DEC.__dict__, "n_layers": 1})
    _, c2 = section_forward(DEC, w, [0, 6], x, keep=True)
    _, ca = section_forward(one, {**w, "layers": w["layers"][:1]}, [0, 6], x, keep=True)
    _, cb = section_forward(one, {**w, "layers": w["layers"][1:]}, [0, 6], ca["y_last"], keep=True)
    assert np.allclose(c2["y_last"], cb["y_last"], atol=1e-14)


def test_gradient_accumulation_over_microbatches(rng):
    """Splitting a batch into micro-batches leaves the summed gradients unchanged
    (the training-equivalence property of paper Sec. 3)."""
    w = make_weights(rng, ENC)
    x, c = rng.standard_normal((11, 8)), rng.standard_normal((11, 8))
    _, cache = section_forward(ENC, w, [0, 4, 7, 11], x, keep=True)
    g_all, _ = section_backward(ENC, w, [0, 4, 7, 11], cache, c)
    _, ca = section_forward(ENC, w, [0, 4], x[:4], keep=True)
    ga, _ = section_backward(ENC, w, [0, 4], ca, c[:4])
    _, cb = section_forward(ENC, w, [0, 3, 7], x[4:], keep=True)
    gb, _ = section_backward(ENC, w, [0, 3, 7], cb, c[4:])
    for name in ["w_qkv", "b_qkv", "w_down", "norm1_g", "norm2_b"]:
        assert np.allclose(g_all["layers"][0][name], ga["layers"][0][name] + gb["layers"][0][name], atol=1e-12)
    assert np.allclose(g_all["final_norm_g"], ga["final_norm_g"] + gb["final_norm_g"], atol=1e-12)


def test_bf16_contract_stays_close_to_fp64_and_is_representable(rng):
    w = make_weights(rng, DEC)
    w = {k: (round_bf16(v) if k != "layers" else [{n: round_bf16(a) for n, a in lw.items()} for lw in v])
         for k, v in w.items()}
    x = round_bf16(rng.standard_normal((7, 8)))
    h64 = section_forward(DEC, w, [0, 7], x)
    hbf = section_forward(DEC, w, [0, 7], x, rnd=round_bf16)
    assert np.array_equal(hbf, round_bf16(hbf))
    assert np.max(np.abs(hbf - h64)) < 0.1 and not np.array_equal(hbf, h64)


def test_distill_step_end_to_end_gradient(rng):
    """d loss / d (student parameter) through KD loss and student stack, by finite differences."""
    t_spec = SectionSpec("decoder", 1, 8, 2, 1, 4, 6, vocab=9, norm_eps=1e-5, rope_base=100.0)
    s_spec = SectionSpec("decoder", 1, 4, 1, 1, 4, 6, vocab=9, norm_eps=1e-5, rope_base=100.0)
    tw, sw = make_weights(rng, t_spec), make_weights(rng, s_spec)
    wt, ws = rng.standard_normal((9, 8)), rng.standard_normal((9, 4))
    cu, ids = [0, 3, 5], np.array([0, 8, 3, 3, 2])
    run = lambda: distill_step(t_spec, tw, s_spec, sw, cu, ids, wt, ws, 2.0, 0.2)
    out = run()
    f = lambda: run()["loss"]
    assert out["loss"] > 0
    assert out["grads"]["layers"][0]["w_up"][2, 1] == pytest.approx(fd_grad(f, sw["layers"][0]["w_up"], (2, 1)), rel=2e-5, abs=1e-9)
    assert out["grads"]["embedding"][3, 2] == pytest.approx(fd_grad(f, sw["embedding"], (3, 2)), rel=2e-5, abs=1e-9)
    assert out["d_w_s"][8, 1] == pytest.approx(fd_grad(f, ws, (8, 1)), rel=2e-5, abs=1e-9)
    g_teacher = fd_grad(f, tw["layers"][0]["w_o"], (0, 0))
    assert g_teacher != 0.0     # the loss depends on the teacher, yet no gradient is produced for it
    assert "teacher_grads" not in out


def test_two_bf16_pipelines_decorrelate_to_rounding_noise():
    """Why chained bf16 results are compared statistically (see parity.assert_parity_chain):
    two runs of the SAME bf16-contract oracle whose only difference is a 1e-6 relative
    perturbation before each rounding (the size of an fp32-vs-fp64 accumulation difference) end
    up differing by whole bf16 ulps on most elements after a few layers."""
    from parity import rel_err, assert_parity_chain
    spec = SectionSpec("decoder", 4, 64, 2, 1, 32, 96, vocab=50, norm_eps=1e-6, rope_base=1e4)
    rng = np.random.default_rng(5)
    w = make_weights(rng, spec, scale=0.05)
    w["embedding"] = 0.05 * w["embedding"]
    rb = lambda t: round_bf16(t)
    w = {k: (rb(v) if k != "layers" else [{n: rb(a) for n, a in lw.items()} for lw in v]) for k, v in w.items()}
    cu, ids = [0, 40, 100, 256], rng.integers(0, 50, 256)
    noise = np.random.default_rng(6)
    pert = lambda t: round_bf16(np.asarray(t) * (1 + 1e-6 * noise.standard_normal(np.shape(t))))
    a = section_forward(spec, w, cu, ids, round_bf16)
    b = section_forward(spec, w, cu, ids, pert)
    e = rel_err(b, a)
    assert np.mean(e > 0) > 0.3                      # not a few isolated flips: a third of all elements differ
    assert 1e-3 < np.sqrt(np.mean(e * e)) < 5e-3     # at the level of a few bf16 roundings
    assert e.max() > 7e-3                            # whole-ulp differences
    assert_parity_chain(b, a, 2e-2, "perturbed bf16 oracle vs bf16 oracle")
