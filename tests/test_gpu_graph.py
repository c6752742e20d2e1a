"""The library allocates nothing and clears memory with kernels only, so a whole distillation step can be
captured into a HIP graph.  Replays are interleaved with eager work and each is checked against the eager result."""
import pytest
import torch

from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_distill_step_replays_from_a_graph():
    work = wl.workload("c2", 0)
    t_cfg = wl.scaled(work.teacher, n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=2, d_ffn=1408, vocab=4096)
    s_cfg = wl.scaled(work.student, n_layers=2, d_model=256, n_q_heads=2, n_kv_heads=2, d_ffn=704, vocab=4096)
    kd = wl.scaled(work.kd, vocab=4096, h_teacher=512, h_student=256, chunk=1024)
    dt, dev = torch.bfloat16, "cuda"
    lengths = [300, 77, 512, 135]
    cu = wl.cu_seqlens_of(lengths)
    n = cu[-1]
    tw, sw = wl.section_weights(t_cfg, 0, "teacher", dev), wl.section_weights(s_cfg, 0, "student", dev)
    wt = wl.normal(0, "lm_head.t", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, dev)
    ws_ = wl.normal(0, "lm_head.s", (kd.vocab, kd.h_student), 0.02, 0.0, dt, dev)
    ids = wl.randint(0, "ids", n, 0, 4096, dev)
    batch = B.Batch(cu)
    ws_t = B.workspace(B.section_workspace_bytes(t_cfg, n, batch.max_seqlen, False), dev, "g.teacher")
    ws_s = B.workspace(B.section_workspace_bytes(s_cfg, n, batch.max_seqlen, True) + B.kd_workspace_bytes(kd, n), dev, "g.student")
    h_t = torch.empty((n, t_cfg.d_model), dtype=dt, device=dev)
    grads = B.zero_grads(sw)
    d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device=dev)
    out = {}

    def step():
        B.section_forward(t_cfg, tw, batch, ids, h_out=h_t, ws=ws_t)
        out.update(B.section_forward_backward(s_cfg, sw, grads, batch, ids, kd=kd, w_teacher=wt, w_student=ws_,
                                              h_teacher=h_t, d_w_student=d_ws, ws=ws_s))

    def zero():
        d_ws.zero_()
        for t in [grads["embedding"], grads["final_norm_g"]] + [v for l in grads["layers"] for v in l.values() if v is not None]:
            t.zero_()

    step()                                                     # eager reference (also warms everything up)
    torch.cuda.synchronize()
    ref_loss, ref_h = out["loss"].clone(), out["h_out"].clone()
    ref_g = grads["layers"][0]["w_qkv"].clone()
    ref_dws = d_ws.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    zero()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        zero()
        # eager work between replays: scribble over the teacher output so that a replay must recompute it
        h_t.fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out["loss"], ref_loss), rep
        assert torch.equal(out["h_out"], ref_h), rep
        # weight gradients go through fp32 atomics (split-K, embedding rows): equal up to summation order
        torch.testing.assert_close(grads["layers"][0]["w_qkv"], ref_g, rtol=1e-4, atol=1e-6)
        torch.testing.assert_close(d_ws, ref_dws, rtol=1e-4, atol=1e-6)
