"""One multimodal micro-batch end to end on the GPU against the oracle chain (Sec. 2.1, Sec. 4.1):
vision-encoder section (forward+backward) -> 4:1 merger + projector -> LLM section fed with embeddings, whose
text rows come from the embedding table and whose image rows come from the merger; the LLM's input gradient
flows back through the merger into the encoder.  Two image samples and one text-only sample."""
import numpy as np
import pytest
import torch

from oracle import round_bf16, round_f32
from oracle.merger import merger_backward, merger_forward
from oracle.section import SectionSpec, section_backward, section_forward
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl
from parity import TOL_BF16, assert_parity_chain, assert_parity_vs_noise, perturbed_rounding

pytestmark = pytest.mark.gpu


def spec_of(cfg):
    return SectionSpec(cfg.arch, cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                       cfg.vocab, cfg.norm_eps, cfg.rope_base)


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def test_vit_merger_llm_chain():
    seed, merge = 11, 4
    vit = wl.scaled(wl.workload("c4", seed).student, n_layers=2, d_model=320, n_q_heads=4, n_kv_heads=4, d_ffn=648)
    llm = wl.scaled(wl.workload("c2", seed).student, n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                    d_ffn=704, vocab=0)
    dt = torch.bfloat16
    patches = [264, 92]                                   # visual tokens of the two image samples (multiples of 4)
    # LLM sequences: [text 7 | image 66 | text 30], [text 41] (text-only sample), [image 23 | text 12]
    llm_lens = [7 + 66 + 30, 41, 23 + 12]
    pos = np.concatenate([7 + np.arange(66), llm_lens[0] + llm_lens[1] + np.arange(23)]).astype(np.int32)
    n_v, n_l = sum(patches), sum(llm_lens)
    vw, lw = wl.section_weights(vit, seed, "vit", "cuda"), wl.section_weights(llm, seed, "llm", "cuda")
    g = lambda tag, shape, std: wl.normal(seed, "chain." + tag, shape, std, 0.0, dt, "cuda")
    mw = dict(w1=g("w1", (640, merge * vit.d_model), 0.02), b1=g("b1", (640,), 0.02), w2=g("w2", (llm.d_model, 640), 0.02),
              b2=g("b2", (llm.d_model,), 0.02))
    x_patch = g("patches", (n_v, vit.d_model), 1.0)
    x_text = g("text_rows", (n_l, llm.d_model), 0.02)     # stands for the embedding gather of the text tokens
    d_out = g("d_h_llm", (n_l, llm.d_model), 1.0)
    cu_v, cu_l = wl.cu_seqlens_of(patches), wl.cu_seqlens_of(llm_lens)
    pos_dev = torch.as_tensor(pos, device="cuda")

    # ---- library: encoder forward (+ backward later needs its own call: run forward-only first for h_vit)
    bv, bl = B.Batch(cu_v), B.Batch(cu_l)
    h_vit = B.section_forward(vit, vw, bv, x_patch)
    ws_m = B.workspace(B.merger_workspace_bytes(mw, len(pos)), "cuda", "merger")
    x_llm = x_text.clone()
    B.merger_forward(mw, h_vit, pos_dev, x_llm, ws_m)
    lg = B.zero_grads(lw)
    out_l = B.section_forward_backward(llm, lw, lg, bl, x_llm, d_h_out=d_out, want_d_x_in=True)
    mg = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in mw.items()}
    d_h_vit = B.merger_backward(mw, mg, h_vit, pos_dev, out_l["d_x_in"], ws_m)
    vg = B.zero_grads(vw)
    out_v = B.section_forward_backward(vit, vw, vg, bv, x_patch, d_h_out=d_h_vit, want_d_x_in=True)
    torch.cuda.synchronize()

    # ---- oracle chain, once with plain rounding and once with a 1e-6 relative jitter in front of every rounding:
    # the second run measures how far two correct bf16 pipelines of this depth drift apart (the noise floor)
    vwr, lwr, mwr = wl.to_f64(vw), wl.to_f64(lw), {k: f64(v) for k, v in mw.items()}

    def oracle_chain(rnd, rnd_res):
        hv, cache_v = section_forward(spec_of(vit), vwr, cu_v, f64(x_patch), rnd, keep=True, rnd_res=rnd_res)
        xl, cache_m = merger_forward(hv, mwr["w1"], mwr["b1"], mwr["w2"], mwr["b2"], pos, f64(x_text), merge, rnd)
        hl, cache_l = section_forward(spec_of(llm), lwr, cu_l, xl, rnd, keep=True, rnd_res=rnd_res)
        gl, d_xl = section_backward(spec_of(llm), lwr, cu_l, cache_l, f64(d_out), rnd, rnd_res=rnd_res)
        d_hv, gm = merger_backward(rnd(d_xl), cache_m, mwr["w1"], mwr["w2"], pos, merge, rnd)
        gv, d_xp = section_backward(spec_of(vit), vwr, cu_v, cache_v, d_hv, rnd, rnd_res=rnd_res)
        return dict(hv=hv, xl=xl, hl=hl, d_xl=d_xl, d_hv=d_hv, d_xp=d_xp, gm=gm, gv=gv, gl=gl)
    r = oracle_chain(round_bf16, round_f32)
    q = oracle_chain(*perturbed_rounding(seed))
    hv, xl, hl, d_xl, d_hv, d_xp, gm, gv, gl = (r[k] for k in ("hv", "xl", "hl", "d_xl", "d_hv", "d_xp", "gm", "gv", "gl"))

    tol = TOL_BF16
    assert_parity_chain(h_vit, hv, tol, "h_vit")
    assert_parity_chain(out_v["h_out"], hv, tol, "h_vit (second pass)")
    assert_parity_chain(x_llm, xl, tol, "LLM input stream")
    assert_parity_chain(out_l["h_out"], hl, tol, "h_llm")
    # backward tensors sit behind the whole chain (encoder, merger, LLM forward, LLM backward, ...): judged against
    # the noise floor of that depth.  Factor 2 rather than 1.5: the attention backward rounds P and dS to bf16 as
    # matrix-core operands, a rounding stage the oracle (and hence its noise floor) does not have.
    assert_parity_vs_noise(out_l["d_x_in"], d_xl, q["d_xl"], "d_x_llm", factor=2.0)
    assert_parity_vs_noise(d_h_vit, d_hv, q["d_hv"], "d_h_vit", factor=2.0)
    assert_parity_vs_noise(out_v["d_x_in"], d_xp, q["d_xp"], "d_patches", factor=2.0)
    for k in mw:
        assert_parity_vs_noise(mg[k], gm[k], q["gm"][k], "merger grad " + k, factor=2.0)
    assert_parity_vs_noise(vg["layers"][0]["w_qkv"], gv["layers"][0]["w_qkv"], q["gv"]["layers"][0]["w_qkv"], "encoder w_qkv grad, first layer", factor=2.0)
    assert_parity_vs_noise(lg["layers"][0]["w_up"], gl["layers"][0]["w_up"], q["gl"]["layers"][0]["w_up"], "LLM w_up grad, first layer", factor=2.0)
    # the text-only sample's rows of the LLM stream are exactly the text rows: it never touched the encoder
    s, e = llm_lens[0], llm_lens[0] + llm_lens[1]
    assert torch.equal(x_llm[s:e], x_text[s:e])
