"""The allocation-free KD entry point (built-in device scratch) against the workspace-taking one.

Two calls in a row on the same GPU, the second on a smaller input: the built-in array keeps the first call's
contents, so the second call only passes if everything that must start from zero is cleared by the call itself.
Collected last (file name) so that a failure here cannot hide the other GPU tests under `pytest -x`.
"""
import pytest
import torch

from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl
from parity import TOL_BF16, TOL_F32, assert_parity

pytestmark = pytest.mark.gpu


def _case(dtype, n, seed):
    kd = wl.KDConfig(2000, 256, 128, 2.0, 512, "bf16" if dtype == torch.bfloat16 else "fp32")
    h_t = wl.normal(seed, "na.ht", (n, kd.h_teacher), 1.0, 0.0, dtype, "cuda")
    h_s = wl.normal(seed, "na.hs", (n, kd.h_student), 1.0, 0.0, dtype, "cuda")
    wt = wl.normal(seed, "na.wt", (kd.vocab, kd.h_teacher), 0.05, 0.0, dtype, "cuda")
    ws = wl.normal(seed, "na.ws", (kd.vocab, kd.h_student), 0.05, 0.0, dtype, "cuda")
    return kd, h_t, h_s, wt, ws


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_call_matches_workspace_call_twice_in_a_row(dtype):
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    for n, seed in ((700, 0), (333, 1)):           # the second call is smaller: stale scratch beyond its rows
        kd, h_t, h_s, wt, ws = _case(dtype, n, seed)
        assert B.kd_workspace_bytes(kd, n) <= B.KD_STATIC_SCRATCH_BYTES
        d_ws_ref = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device="cuda")
        ref = B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws_ref)
        # outputs are the caller's, allocated before the call
        loss = torch.full((), -1.0, dtype=torch.float32, device="cuda")
        kl = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
        d_h = torch.full_like(h_s, 7.0)
        d_ws = torch.zeros_like(d_ws_ref)
        B.kd_loss_forward_backward_static(kd, wt, ws, h_t, h_s, loss, kl, d_h, d_ws)
        torch.cuda.synchronize()
        # same kernels on the same inputs: everything without floating-point atomics is bit-identical
        assert torch.equal(loss, ref["loss"]), (n, loss.item(), ref["loss"].item())
        assert torch.equal(kl, ref["kl_tok"]), n
        assert torch.equal(d_h, ref["d_h_s"]), n
        assert_parity(d_ws, d_ws_ref.double().cpu().numpy(), tol, f"d_w_s n={n}")       # split-K sums: order differs
        assert float(loss.item()) > 0


def test_static_scratch_call_rejects_sizes_beyond_its_buffer():
    n = 8192                                        # [8192, 2000] fp32 logits twice: beyond 64 MiB
    kd, h_t, h_s, wt, ws = _case(torch.bfloat16, n, 2)
    big = wl.scaled(kd, chunk=2000)
    assert B.kd_workspace_bytes(big, n) > B.KD_STATIC_SCRATCH_BYTES
    out = torch.zeros(n, dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError, match="built-in buffer"):
        B.kd_loss_forward_backward_static(big, wt, ws, h_t, h_s, out, out, None)
