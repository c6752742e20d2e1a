"""Parity at the full workload sizes, in the launch configuration bench.py times.

The oracle cannot run 16 K .. 92 K tokens of these models in test time, so it runs what it can compute
exactly: whole SEQUENCES sampled from the packed batch -- the shortest ones AND a long one (c2: its longest, 4096
tokens; c4: its longest, 4038; c5: 5418 tokens for the student stack) -- because a sequence's outputs and input
gradients depend only on its own tokens ("packed == each sequence alone" is one of the oracle's pins), and sampled
TOKENS for the distillation loss (tokens are independent there).  Three kinds of checks:
  * rows of the FULL-batch run against the oracle on the sampled sequences (forward outputs, per-token KL);
  * every gradient (all weight gradients, embedding rows, lm_head gradient, input gradient) of a micro-batch made of
    the sampled sequences against the oracle on that micro-batch, at full model width and vocabulary;
  * size-independent properties on the full batch: the sampled sequences come out bit-identical whether they run
    packed in the full batch or in their own micro-batch (includes the longest sequence), gradient accumulation over
    micro-batches equals the full batch, loss == loss_scale * sum(kl_tok), KL >= 0, softmax-difference gradients
    summing to zero over the vocabulary.
Each kernel on its own is held to the strict per-element bound at these shapes in test_gpu_fullshape_kernels.py.

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
    return uniq, inv, wl.to_f64(table[torch.as_tensor(uniq, device=table.device)])


def seq_ranges(cu):
    return sorted((cu[i + 1] - cu[i], cu[i], cu[i + 1]) for i in range(len(cu) - 1) if cu[i + 1] > cu[i])


def sampled(cu, n_short, long_len=None):
    """(lo, hi) of the n_short shortest sequences and of the longest (or the one of length long_len)."""
    r = seq_ranges(cu)
    pick = r[:n_short] + ([r[-1]] if long_len is None else [x for x in r if x[0] == long_len])
    return [(lo, hi) for _, lo, hi in pick]


def gather_rows(t, ranges):
    return torch.cat([t[lo:hi] for lo, hi in ranges]).contiguous()


def noise_check(gpu, ref, alt, name):
    print(assert_parity_vs_noise(gpu, ref, alt, name))


def grads_vs_noise(grads, ref, alt, prefix):
    for k, v in ref.items():
        if k == "layers":
            for li, lw in enumerate(v):
                for nme, r in lw.items():
                    if r is not None:
                        noise_check(grads["layers"][li][nme], r, alt["layers"][li][nme], f"{prefix} l{li}.{nme}")
        elif v is not None and k != "embedding":
            noise_check(grads[k], v, alt[k], f"{prefix} {k}")


def oracle_decoder_inputs(cfg, w, ids_sub):
    """fp64 weights with the embedding table compacted to the rows the micro-batch uses."""
    wf = dict(wl.to_f64({k: v for k, v in w.items() if k != "embedding"}))
    uniq, inv, table = compact_ids(ids_sub.cpu().numpy(), w["embedding"])
    wf["embedding"] = table
    spec = spec_of(cfg)
    spec.vocab = table.shape[0]
    return spec, wf, inv, uniq


@pytest.mark.parametrize("name,n_short,long_len", [("c2", 2, None), ("c5", 2, 5418)])
def test_full_size_distill_step_on_sampled_sequences(name, n_short, long_len):
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
    # ---- size-independent properties of the full batch
    kl = out["kl_tok"].double()
    assert torch.isfinite(kl).all() and float(kl.min()) > -1e-5
    assert abs(out["loss"].item() - float(kl.sum()) / n) <= 1e-5 * abs(out["loss"].item())
    assert torch.isfinite(d_ws).all() and float(d_ws.abs().max()) > 0
    col = d_ws.double().sum(dim=0)                                  # sum_v dz[t, v] = 0  =>  column sums vanish
    assert float(col.abs().max()) <= 1e-3 * float(d_ws.double().abs().sum(dim=0).max())
    for g in grads["layers"]:
        assert all(torch.isfinite(t).all() and float(t.abs().max()) > 0 for t in g.values() if t is not None)
    # ---- the sampled sequences (shortest ones and a long one) as a micro-batch of their own
    short = sampled(cu, n_short, 0)                                 # long_len = 0 matches nothing: the short ones only
    longest = sampled(cu, 0)                                        # the longest sequence of the batch
    ranges = short + longest
    cu_sub = wl.cu_seqlens_of([hi - lo for lo, hi in ranges])
    ids_sub, b_sub = gather_rows(ids, ranges), B.Batch(cu_sub)
    ht_sub = B.section_forward(t_cfg, tw, b_sub, ids_sub)
    g_sub = B.zero_grads(sw)
    dws_sub = torch.zeros_like(d_ws)
    out_sub = B.section_forward_backward(s_cfg, sw, g_sub, b_sub, ids_sub, kd=kd, w_teacher=wt, w_student=ws, h_teacher=ht_sub,
                                         d_w_student=dws_sub, loss_scale=1.0 / n)
    torch.cuda.synchronize()
    # packed == each sequence in another micro-batch, bit for bit, at the longest sequence of the workload too
    assert torch.equal(ht_sub, gather_rows(h_t, ranges)), "teacher rows differ between the full batch and the micro-batch"
    assert torch.equal(out_sub["h_out"], gather_rows(out["h_out"], ranges))
    assert torch.equal(out_sub["kl_tok"], gather_rows(out["kl_tok"], ranges))
    # ---- oracle on what it can afford: c2 the whole micro-batch (incl. the 4096-token sequence), c5 the short ones
    # for the full step and one 5418-token sequence for the student stack alone
    o_ranges = ranges if long_len is None else short
    n_o = sum(hi - lo for lo, hi in o_ranges)
    cu_o = wl.cu_seqlens_of([hi - lo for lo, hi in o_ranges])
    ids_o = gather_rows(ids, o_ranges)
    t_spec, t_wf, t_inv, _ = oracle_decoder_inputs(t_cfg, tw, ids_o)
    s_spec, s_wf, s_inv, s_uniq = oracle_decoder_inputs(s_cfg, sw, ids_o)
    wt64, ws64 = wl.to_f64(wt), wl.to_f64(ws)
    runs = []
    for rnd, rnd_res in ((round_bf16, round_f32), perturbed_rounding(n_o)):
        ht = section_forward(t_spec, t_wf, cu_o, t_inv, rnd, rnd_res=rnd_res)
        hs, cache = section_forward(s_spec, s_wf, cu_o, s_inv, rnd, keep=True, rnd_res=rnd_res)
        k = oracle_kd(ht, hs, wt64, ws64, kd.temperature, 1.0 / n, rnd, token_block=512)
        g, _ = section_backward(s_spec, s_wf, cu_o, cache, k["d_h_s"], rnd)
        runs.append(dict(ht=ht, hs=hs, kd=k, g=g))
    ref, alt = runs
    noise_check(gather_rows(h_t, o_ranges), ref["ht"], alt["ht"], "h_teacher rows of the full batch")
    noise_check(gather_rows(out["h_out"], o_ranges), ref["hs"], alt["hs"], "h_student rows of the full batch")
    noise_check(gather_rows(out["kl_tok"], o_ranges), ref["kd"]["kl_tok"], alt["kd"]["kl_tok"], "kl_tok rows of the full batch")
    if long_len is None:
        # every gradient of the micro-batch (the GPU ran exactly the oracle's sequences)
        grads_vs_noise(g_sub, ref["g"], alt["g"], "micro-batch grad")
        noise_check(dws_sub, ref["kd"]["d_w_s"], alt["kd"]["d_w_s"], "micro-batch d_w_student")
        emb = g_sub["embedding"][torch.as_tensor(s_uniq, device="cuda")]
        noise_check(emb, ref["g"]["embedding"], alt["g"]["embedding"], "micro-batch embedding rows")
    else:
        # c5: gradients of the short sequences alone, then the student stack on one long sequence
        g_s = B.zero_grads(sw)
        dws_s = torch.zeros_like(d_ws)
        b_s = B.Batch(cu_o)
        ht_s = B.section_forward(t_cfg, tw, b_s, ids_o)
        B.section_forward_backward(s_cfg, sw, g_s, b_s, ids_o, kd=kd, w_teacher=wt, w_student=ws, h_teacher=ht_s,
                                   d_w_student=dws_s, loss_scale=1.0 / n)
        torch.cuda.synchronize()
        grads_vs_noise(g_s, ref["g"], alt["g"], "micro-batch grad")
        noise_check(dws_s, ref["kd"]["d_w_s"], alt["kd"]["d_w_s"], "micro-batch d_w_student")
        emb = g_s["embedding"][torch.as_tensor(s_uniq, device="cuda")]
        noise_check(emb, ref["g"]["embedding"], alt["g"]["embedding"], "micro-batch embedding rows")
        (lo, hi), = sampled(cu, 0, long_len)
        spec, wf, inv, _ = oracle_decoder_inputs(s_cfg, sw, ids[lo:hi])
        hs_ref = section_forward(spec, wf, [0, hi - lo], inv, round_bf16, rnd_res=round_f32)
        prnd, prnd_res = perturbed_rounding(lo)
        hs_alt = section_forward(spec, wf, [0, hi - lo], inv, prnd, rnd_res=prnd_res)
        noise_check(out["h_out"][lo:hi], hs_ref, hs_alt, f"h_student[{lo}:{hi}] ({hi - lo} tokens)")


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
    # ---- gradient accumulation over two micro-batches of whole samples == the one packed batch (same sequences,
    # same per-token values; only the fp32 summation order of the weight gradients differs)
    half = cu[len(cu) // 2]
    g2 = B.zero_grads(w)
    for lo, hi, c in ((0, half, cu[:len(cu) // 2 + 1]), (half, n, [v - half for v in cu[len(cu) // 2:]])):
        o2 = B.section_forward_backward(cfg, w, g2, B.Batch(c), x[lo:hi].contiguous(), d_h_out=d_h[lo:hi].contiguous(), want_d_x_in=True)
        assert torch.equal(o2["h_out"], out["h_out"][lo:hi]) and torch.equal(o2["d_x_in"], out["d_x_in"][lo:hi])
    torch.cuda.synchronize()
    for li in (0, 7):
        for nme, t in grads["layers"][li].items():
            assert_parity(g2["layers"][li][nme], t.double().cpu().numpy(), 2e-4, f"accumulated l{li}.{nme}")
    # ---- the two shortest samples and the longest one (4038 patches): forward rows and input gradient of the full
    # batch, and every weight gradient of a micro-batch made of these samples, against the oracle
    ranges = sampled(cu, 2)
    cu_sub = wl.cu_seqlens_of([hi - lo for lo, hi in ranges])
    x_sub, dh_sub = gather_rows(x, ranges), gather_rows(d_h, ranges)
    g_sub = B.zero_grads(w)
    out_sub = B.section_forward_backward(cfg, w, g_sub, B.Batch(cu_sub), x_sub, d_h_out=dh_sub, want_d_x_in=True)
    torch.cuda.synchronize()
    assert torch.equal(out_sub["h_out"], gather_rows(out["h_out"], ranges))
    assert torch.equal(out_sub["d_x_in"], gather_rows(out["d_x_in"], ranges))
    spec, wf = spec_of(cfg), wl.to_f64(w)
    runs = []
    for rnd, rnd_res in ((round_bf16, round_f32), perturbed_rounding(17)):
        h, cache = section_forward(spec, wf, cu_sub, wl.to_f64(x_sub), rnd, keep=True, rnd_res=rnd_res)
        g, dx = section_backward(spec, wf, cu_sub, cache, wl.to_f64(dh_sub), rnd)
        runs.append((h, dx, g))
    (h_ref, dx_ref, g_ref), (h_alt, dx_alt, g_alt) = runs
    noise_check(out_sub["h_out"], h_ref, h_alt, "h_out (2 shortest + longest sample)")
    noise_check(out_sub["d_x_in"], dx_ref, dx_alt, "d_x_in (2 shortest + longest sample)")
    grads_vs_noise(g_sub, g_ref, g_alt, "micro-batch grad")


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
