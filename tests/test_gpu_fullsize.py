"""Parity at the full workload sizes, in the launch configuration bench.py times.

The oracle cannot run 16 K .. 92 K tokens of these models in test time, so it runs what it can compute
exactly: whole SEQUENCES sampled from the packed batch (a sequence's outputs and input gradients depend
only on its own tokens: "packed == each sequence alone" is one of the oracle's pins), and sampled TOKENS
for the distillation loss (tokens are independent there).  Size-independent properties cover the rest:
loss == loss_scale * sum(kl_tok), KL >= 0, softmax-difference gradients summing to zero over the vocabulary.
Weight gradients are compared element-wise at reduced width in test_gpu_section.py.

Outputs of the deep full-width stacks are held to the measured bf16 noise floor (parity.assert_parity_vs_noise):
the oracle is run a second time with 1e-6 relative perturbations before every rounding, and the HIP result
may deviate from the oracle by at most 1.5 x what that second oracle run does.
"""
import numpy as np
import pytest
import torch

from oracle import round_bf16, round_f32
from oracle.kd import kd_loss_forward_backward as oracle_kd
from oracle.section import section_backward, section_forward
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl
from parity import TOL_BF16, TOL_LOSS_BF16, assert_kl_tok, assert_parity, assert_parity_chain, assert_parity_vs_noise, perturbed_rounding
from test_gpu_section import spec_of

pytestmark = pytest.mark.gpu


def compact_ids(ids_np, table):
    """Embedding rows actually used, so the oracle does not need the whole fp64 table."""
    uniq, inv = np.unique(ids_np, return_inverse=True)
    return inv, wl.to_f64(table[torch.as_tensor(uniq, device=table.device)])


def oracle_section_on_sequence(cfg, w, ids_or_x, lo, hi):
    spec = spec_of(cfg)
    wf = {k: v for k, v in wl.to_f64({k: v for k, v in w.items() if k != "embedding"}).items()}
    if cfg.vocab > 0:
        inv, table = compact_ids(ids_or_x[lo:hi].cpu().numpy(), w["embedding"])
        wf["embedding"] = table
        spec.vocab = table.shape[0]
        x = inv
    else:
        x = wl.to_f64(ids_or_x[lo:hi])
    return spec, wf, x


def shortest_sequences(cu, k):
    lens = [(cu[i + 1] - cu[i], i) for i in range(len(cu) - 1) if cu[i + 1] > cu[i]]
    return [(cu[i], cu[i + 1]) for _, i in sorted(lens)[:k]]


@pytest.mark.parametrize("name,n_seqs", [("c2", 3), ("c5", 2)])
def test_full_size_distill_step_on_sampled_sequences(name, n_seqs):
    work = wl.workload(name, 0)
    t_cfg, s_cfg, kd = work.teacher, work.student, work.kd
    dt = torch.bfloat16
    tw, sw = wl.section_weights(t_cfg, 0, "teacher", "cuda"), wl.section_weights(s_cfg, 0, "student", "cuda")
    wt = wl.normal(0, "lm_head.t", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, "cuda")
    ws = wl.normal(0, "lm_head.s", (kd.vocab, kd.h_student), 0.02, 0.0, dt, "cuda")
    cu = wl.cu_seqlens_of(work.lengths)
    n = cu[-1]
    assert n == work.n_tokens
    ids = wl.randint(0, "ids", n, 0, t_cfg.vocab, "cuda")
    batch = B.Batch(cu)
    h_t = B.section_forward(t_cfg, tw, batch, ids)
    grads = B.zero_grads(sw)
    d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device="cuda")
    out = B.section_forward_backward(s_cfg, sw, grads, batch, ids, kd=kd, w_teacher=wt, w_student=ws, h_teacher=h_t,
                                     d_w_student=d_ws)
    torch.cuda.synchronize()
    # size-independent properties
    kl = out["kl_tok"].double()
    assert torch.isfinite(kl).all() and float(kl.min()) > -1e-5
    assert abs(out["loss"].item() - float(kl.sum()) / n) <= 1e-5 * abs(out["loss"].item())
    assert torch.isfinite(d_ws).all() and float(d_ws.abs().max()) > 0
    col = d_ws.double().sum(dim=0)                                  # sum_v dz[t, v] = 0  =>  column sums vanish
    assert float(col.abs().max()) <= 1e-3 * float(d_ws.double().abs().sum(dim=0).max())
    for g in grads["layers"]:
        assert all(torch.isfinite(t).all() and float(t.abs().max()) > 0 for t in g.values() if t is not None)
    # sampled whole sequences against the oracle
    wt64, ws64 = wl.to_f64(wt), wl.to_f64(ws)
    for lo, hi in shortest_sequences(cu, n_seqs):
        prnd, prnd_res = perturbed_rounding(lo)
        spec, wf, x = oracle_section_on_sequence(t_cfg, tw, ids, lo, hi)
        ht_ref = section_forward(spec, wf, [0, hi - lo], x, round_bf16, rnd_res=round_f32)
        ht_alt = section_forward(spec, wf, [0, hi - lo], x, prnd, rnd_res=prnd_res)
        print(assert_parity_vs_noise(h_t[lo:hi], ht_ref, ht_alt, f"h_teacher[{lo}:{hi}]"))
        spec, wf, x = oracle_section_on_sequence(s_cfg, sw, ids, lo, hi)
        hs_ref = section_forward(spec, wf, [0, hi - lo], x, round_bf16, rnd_res=round_f32)
        hs_alt = section_forward(spec, wf, [0, hi - lo], x, prnd, rnd_res=prnd_res)
        print(assert_parity_vs_noise(out["h_out"][lo:hi], hs_ref, hs_alt, f"h_student[{lo}:{hi}]"))
        ref = oracle_kd(ht_ref, hs_ref, wt64, ws64, kd.temperature, 1.0 / n, round_bf16, need_grad=False)
        alt = oracle_kd(ht_alt, hs_alt, wt64, ws64, kd.temperature, 1.0 / n, prnd, need_grad=False)
        print(assert_parity_vs_noise(out["kl_tok"][lo:hi], ref["kl_tok"], alt["kl_tok"], f"kl_tok[{lo}:{hi}]"))


def test_full_size_c4_encoder_on_sampled_samples():
    work = wl.workload("c4", 0)
    cfg = work.student
    order, offs, cus = B.pack_microbatches(work.lengths, 1 << 30, 0)     # text-only samples are dropped here
    assert len(order) == 45 and len(cus) == 1
    cu = cus[0]
    n = cu[-1]
    w = wl.section_weights(cfg, 0, "vit", "cuda")
    x = wl.normal(0, "patches", (n, cfg.d_model), 1.0, 0.0, torch.bfloat16, "cuda")
    d_h = wl.normal(0, "d_h_out", (n, cfg.d_model), 1.0, 0.0, torch.bfloat16, "cuda")
    grads = B.zero_grads(w)
    out = B.section_forward_backward(cfg, w, grads, B.Batch(cu), x, d_h_out=d_h, want_d_x_in=True)
    torch.cuda.synchronize()
    for g in grads["layers"]:
        assert all(torch.isfinite(t).all() and float(t.abs().max()) > 0 for t in g.values())
    for lo, hi in shortest_sequences(cu, 2):
        prnd, prnd_res = perturbed_rounding(lo)
        spec, wf, xs = oracle_section_on_sequence(cfg, w, x, lo, hi)
        h_ref, cache = section_forward(spec, wf, [0, hi - lo], xs, round_bf16, keep=True, rnd_res=round_f32)
        _, dx_ref = section_backward(spec, wf, [0, hi - lo], cache, wl.to_f64(d_h[lo:hi]), round_bf16)
        h_alt, cache_alt = section_forward(spec, wf, [0, hi - lo], xs, prnd, keep=True, rnd_res=prnd_res)
        _, dx_alt = section_backward(spec, wf, [0, hi - lo], cache_alt, wl.to_f64(d_h[lo:hi]), prnd)
        print(assert_parity_vs_noise(out["h_out"][lo:hi], h_ref, h_alt, f"h_out[{lo}:{hi}]"))
        print(assert_parity_vs_noise(out["d_x_in"][lo:hi], dx_ref, dx_alt, f"d_x_in[{lo}:{hi}]"))


def c3_inputs(n):
    kd = wl.workload("c3", 0).kd
    dt = torch.bfloat16
    h_t = wl.normal(0, "c3.ht", (n, kd.h_teacher), 1.0, 0.0, dt, "cuda")
    h_s = wl.normal(0, "c3.hs", (n, kd.h_student), 1.0, 0.0, dt, "cuda")
    wt = wl.normal(0, "c3.wt", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, "cuda")
    ws = wl.normal(0, "c3.ws", (kd.vocab, kd.h_student), 0.02, 0.0, dt, "cuda")
    return kd, h_t, h_s, wt, ws


def test_c3_full_vocab_reduced_tokens_every_output():
    """Full vocabulary 151936 in 19 chunks (last one 4480 wide), full hidden sizes, 384 tokens: the oracle covers all outputs."""
    n = 384
    kd, h_t, h_s, wt, ws = c3_inputs(n)
    d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device="cuda")
    out = B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws)
    ref = oracle_kd(wl.to_f64(h_t), wl.to_f64(h_s), wl.to_f64(wt), wl.to_f64(ws), kd.temperature, 1.0 / n, round_bf16,
                    token_block=128)
    assert abs(out["loss"].item() - ref["loss"]) <= TOL_LOSS_BF16 * ref["loss"]
    assert_kl_tok(out["kl_tok"], ref["kl_tok"], TOL_LOSS_BF16, kd.vocab)
    assert_parity(out["d_h_s"], ref["d_h_s"], TOL_BF16, "d_h_s")
    assert_parity(d_ws, ref["d_w_s"], TOL_BF16, "d_w_s")


def test_c3_full_size_sampled_tokens_and_properties():
    n = 8192
    kd, h_t, h_s, wt, ws = c3_inputs(n)
    d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device="cuda")
    out = B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws)
    torch.cuda.synchronize()
    kl = out["kl_tok"].double()
    assert float(kl.min()) > 0 and abs(out["loss"].item() - float(kl.sum()) / n) <= 1e-5 * out["loss"].item()
    col = d_ws.double().sum(dim=0)
    assert float(col.abs().max()) <= 1e-3 * float(d_ws.double().abs().sum(dim=0).max())
    tok = wl.randint(1, "c3.sample", 96, 0, n).long().cuda()
    ref = oracle_kd(wl.to_f64(h_t[tok]), wl.to_f64(h_s[tok]), wl.to_f64(wt), wl.to_f64(ws), kd.temperature, 1.0 / n,
                    round_bf16)
    assert_kl_tok(out["kl_tok"][tok], ref["kl_tok"], TOL_LOSS_BF16, kd.vocab, "kl_tok (sampled tokens)")
    assert_parity(out["d_h_s"][tok], ref["d_h_s"], TOL_BF16, "d_h_s (sampled tokens)")
