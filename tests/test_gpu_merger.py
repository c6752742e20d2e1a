"""Vision -> language hand-off on the GPU against the oracle (Sec. 2.1, Sec. 4.1)."""
import numpy as np
import pytest
import torch

from oracle import identity, round_bf16
from oracle.merger import merger_backward, merger_forward
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl
from parity import TOL_BF16, TOL_F32, assert_parity, assert_parity_chain

pytestmark = pytest.mark.gpu


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


@pytest.mark.parametrize("dtype,groups,dv,dh,dl,n_llm", [
    (torch.bfloat16, 1000, 1280, 5120, 2048, 5000),      # c4's encoder width, several tiles, ragged group count
    (torch.bfloat16, 37, 64, 136, 72, 50),               # widths off the 64-multiples: generic GEMM path
    (torch.float32, 129, 32, 48, 40, 300)])
def test_merger_forward_backward(dtype, groups, dv, dh, dl, n_llm):
    merge = 4
    rnd = round_bf16 if dtype == torch.bfloat16 else identity
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    g = lambda tag, shape, std: wl.normal(5, "merger." + tag, shape, std, 0.0, dtype, "cuda")
    w = dict(w1=g("w1", (dh, merge * dv), 0.02), b1=g("b1", (dh,), 0.02), w2=g("w2", (dl, dh), 0.02), b2=g("b2", (dl,), 0.02))
    h = g("h", (merge * groups, dv), 1.0)
    x0 = g("x", (n_llm, dl), 1.0)
    d_x = g("dx", (n_llm, dl), 1.0)
    # image positions: a seeded subset of the LLM stream, in increasing order as in a packed sample
    pos = torch.sort(wl.uniform(5, "merger.pos", n_llm).argsort()[:groups]).values.to(torch.int32).cuda()
    ws = B.workspace(B.merger_workspace_bytes(w, groups), "cuda", "merger")
    x = x0.clone()
    B.merger_forward(w, h, pos, x, ws)
    grads = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in w.items()}
    d_h = B.merger_backward(w, grads, h, pos, d_x, ws)
    wr = {k: f64(v) for k, v in w.items()}
    pr = pos.cpu().numpy()
    xr, cache = merger_forward(f64(h), wr["w1"], wr["b1"], wr["w2"], wr["b2"], pr, f64(x0), merge, rnd)
    dhr, gr = merger_backward(f64(d_x), cache, wr["w1"], wr["w2"], pr, merge, rnd)
    text = np.setdiff1d(np.arange(n_llm), pr)
    assert torch.equal(x[torch.as_tensor(text, device="cuda")], x0[torch.as_tensor(text, device="cuda")])   # text rows untouched
    chain = assert_parity_chain if dtype == torch.bfloat16 else assert_parity
    chain(x[pos.long()], xr[pr], tol, "projected rows")
    chain(d_h, dhr, tol, "d_h_vit")
    for k in ("w1", "b1", "w2", "b2"):
        chain(grads[k], gr[k], tol if dtype == torch.bfloat16 else 2e-4, "grad " + k)


def test_merger_text_only_batch_and_out_of_range_positions():
    w = {k: torch.zeros(s, dtype=torch.bfloat16, device="cuda") for k, s in dict(w1=(16, 32), b1=(16,), w2=(8, 16), b2=(8,)).items()}
    w["b2"] += 1.0
    ws = B.workspace(B.merger_workspace_bytes(w, 4), "cuda", "merger")
    x = torch.zeros((6, 8), dtype=torch.bfloat16, device="cuda")
    empty = torch.empty((0, 8), dtype=torch.bfloat16, device="cuda")
    B.merger_forward(w, empty, torch.empty(0, dtype=torch.int32, device="cuda"), x, ws)          # encoder skipped
    assert float(x.abs().max()) == 0.0
    h = torch.ones((16, 8), dtype=torch.bfloat16, device="cuda")
    pos = torch.tensor([0, 99, -1, 5], dtype=torch.int32, device="cuda")                         # two rows off the stream
    B.merger_forward(w, h, pos, x, ws)
    torch.cuda.synchronize()
    assert torch.all(x[0] == 1.0) and torch.all(x[5] == 1.0) and float(x[1:5].abs().max()) == 0.0
