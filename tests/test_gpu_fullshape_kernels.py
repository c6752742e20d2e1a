"""Kernel-level parity at the real shapes of the workloads, strict per-element criterion.

Each test hands ONE kernel (through the C ABI, with the library's own automatic tile / split-K choice) seeded inputs
that the oracle receives as well, at the M / N / K, sequence lengths and head shapes of workloads c2, c4 and c5, and
compares element by element: every output element for the attention cases (one KV group is seconds of dense fp64
work), sampled output rows for the GEMM roles (an output row needs the whole K extent of its operands, which the
oracle computes exactly; the rows are spread over every workgroup tile and include the first and last ones).
"""
import numpy as np
import pytest
import torch

from oracle import ops, round_bf16
from oracle.attention import attention_bwd, attention_fwd
from oracle.kd import kd_loss_forward_backward as oracle_kd
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl
from parity import TOL_BF16, TOL_F32, TOL_LOSS_BF16, assert_kl_tok, assert_parity, assert_parity_rows

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def dev(name, shape, std=1.0, dtype=BF):
    return wl.normal(11, name, shape, std, 0.0, dtype, "cuda")


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def sample_rows(m, k=768, seed=5):
    """Sorted row sample: k random rows plus the first and last eight (first tile, ragged last tile)."""
    r = np.random.default_rng(seed).choice(m, size=min(k, m), replace=False)
    return np.unique(np.concatenate([r, np.arange(min(8, m)), np.arange(max(0, m - 8), m)]))


# ---------------------------------------------------------------------------------------------- attention
# (nq, nkv, hd, causal, L): one KV group of c2 / c5 (GQA 4:1, hd 128, causal) at the longest c2 sequence and the longest
# c5 sequence, and two heads of the c4 encoder (hd 80, bidirectional) at its longest sample
LONG_ATT = [(4, 1, 128, True, 4096), (4, 1, 128, True, 10687), (2, 2, 80, False, 4038)]


@pytest.mark.parametrize("nq,nkv,hd,causal,L", LONG_ATT)
def test_attention_long_sequence_forward_backward(nq, nkv, hd, causal, L):
    # a short neighbour on each side: the long sequence neither starts at row 0 nor ends the batch
    cu = [0, 37, 37 + L, 37 + L + 150]
    n = cu[-1]
    batch = B.Batch(cu)
    qkv = dev(f"lq{L}", (n, (nq + 2 * nkv) * hd))
    d_o = dev(f"ldo{L}", (n, nq * hd))
    x = f64(qkv)
    q = x[:, :nq * hd].reshape(n, nq, hd)
    k = x[:, nq * hd:(nq + nkv) * hd].reshape(n, nkv, hd)
    v = x[:, (nq + nkv) * hd:].reshape(n, nkv, hd)
    o, lse = B.k_attention_forward(qkv, batch, nq, nkv, hd, causal)
    o_ref, lse_ref = attention_fwd(q, k, v, cu, causal, return_lse=True)
    o_ref = round_bf16(o_ref)
    # rows of very different scale in one tensor (13 keys ... 10687 keys): per-row error floor, see parity.py
    print("o", assert_parity_rows(o, o_ref.reshape(n, -1), TOL_BF16, "o"), "lse", assert_parity(lse, lse_ref, 1e-3, "lse"))
    # backward from the oracle's stored output and log-sum-exp (identical inputs on both sides); the oracle rounds P
    # and dS where they become matrix-product operands, as a path with bf16 matrix units does
    o_in = torch.tensor(o_ref.reshape(n, -1), dtype=BF, device="cuda")
    lse_in = torch.tensor(lse_ref, dtype=torch.float32, device="cuda")
    dq, dk, dv = attention_bwd(f64(d_o).reshape(n, nq, hd), q, k, v, cu, causal, o=o_ref, rnd_p=round_bf16)
    dqkv = B.k_attention_backward(qkv, o_in, lse_in, d_o, batch, nq, nkv, hd, causal)
    for name, ref, sl in [("dq", dq, slice(0, nq * hd)), ("dk", dk, slice(nq * hd, (nq + nkv) * hd)),
                          ("dv", dv, slice((nq + nkv) * hd, None))]:
        print(name, assert_parity_rows(dqkv[:, sl], round_bf16(ref.reshape(n, -1)), TOL_BF16, name))


# ---------------------------------------------------------------------------------------------- GEMM roles
def _check_rows(c, ref_rows, rows, tol, name):
    got = c[torch.as_tensor(rows, device=c.device)]
    # the error floor is the rms of the compared rows (a sample of the whole output)
    print(name, assert_parity(got, ref_rows, tol, name))


# (name, M, N, K, bias, fp32 residual): forward linears  y[M,N] = x[M,K] W[N,K]^T
FPROP = [("c2 teacher gate/up as a plain GEMM", 16384, 11008, 2048, False, False),
         ("c5 teacher down-projection + fp32 residual", 32768, 4096, 11008, False, True),
         ("c5 student qkv", 32768, 2048, 1536, False, False),
         ("c4 fc1 + bias, ragged M", 92346, 5120, 1280, True, False)]


@pytest.mark.parametrize("name,M,N,K,bias,res", FPROP, ids=[c[0] for c in FPROP])
def test_gemm_forward_roles_at_full_shape(name, M, N, K, bias, res):
    x, w = dev("gx" + name, (M, K)), dev("gw" + name, (N, K), 0.02)
    b = dev("gb" + name, (N,), 0.02) if bias else None
    r = dev("gr" + name, (M, N), 1.0, torch.float32) if res else None
    c = B.k_gemm(x, w, bias=b, residual=r, c_fp32=res)
    rows = sample_rows(M)
    ref = f64(x[torch.as_tensor(rows, device="cuda")]) @ f64(w).T
    if bias:
        ref = ref + f64(b)[None, :]
    if res:
        ref = ref + f64(r[torch.as_tensor(rows, device="cuda")])
    _check_rows(c, ref if res else round_bf16(ref), rows, TOL_F32 if res else TOL_BF16, name)


# input gradients  dx[M,N] = dy[M,K] W[K,N]  (W stored [out = K, in = N]: the K-major "B" operand)
DGRAD = [("c2 teacher-shaped up-projection dgrad", 16384, 2048, 11008), ("c5 student down-projection dgrad", 32768, 8960, 1536),
         ("c4 fc2 dgrad, ragged M", 92346, 5120, 1280)]


@pytest.mark.parametrize("name,M,N,K", DGRAD, ids=[c[0] for c in DGRAD])
def test_gemm_dgrad_roles_at_full_shape(name, M, N, K):
    dy, w = dev("dgy" + name, (M, K)), dev("dgw" + name, (K, N), 0.02)
    c = B.k_gemm(dy, w, False, True)
    rows = sample_rows(M)
    ref = f64(dy[torch.as_tensor(rows, device="cuda")]) @ f64(w)
    _check_rows(c, round_bf16(ref), rows, TOL_BF16, name)


# weight gradients  dW[out, in] += dy[n, out]^T x[n, in]: both operands K-major, reduction over the tokens, fp32
# accumulation into the caller's buffer, split-K chosen by the library
WGRAD = [("c2 student up-projection, K = 16384", 5632, 1024, 16384), ("c2 teacher-shaped, K = 16384", 11008, 2048, 16384),
         ("c5 student up-projection, K = 32768", 17920, 1536, 32768), ("c4 fc1, K = 92346 (ragged)", 5120, 1280, 92346),
         ("c5 student o-projection, K = 32768", 1536, 1536, 32768)]


@pytest.mark.parametrize("name,out,inn,K", WGRAD, ids=[c[0] for c in WGRAD])
def test_gemm_wgrad_roles_at_full_shape(name, out, inn, K):
    dy, x = dev("wgy" + name, (K, out)), dev("wgx" + name, (K, inn))
    dw0 = dev("wg0" + name, (out, inn), 3.0, torch.float32)             # accumulated into, not overwritten
    dw = dw0.clone()
    B.k_gemm(dy, x, True, True, c=dw, c_fp32=True, accumulate=True, split_k=0)
    rows = sample_rows(out, 512)
    ridx = torch.as_tensor(rows, device="cuda")
    ref = f64(dw0[ridx]) + f64(dy[:, ridx]).T @ f64(x)
    _check_rows(dw, ref, rows, TOL_F32, name)


SWIGLU = [("c2 teacher", 16384, 5504, 2048), ("c2 student", 16384, 2816, 1024), ("c5 student", 32768, 8960, 1536)]


@pytest.mark.parametrize("name,M,F,K", SWIGLU, ids=[c[0] for c in SWIGLU])
def test_gemm_swiglu_epilogue_at_full_shape(name, M, F, K):
    x, w = dev("sx" + name, (M, K)), dev("sw" + name, (2 * F, K), 0.02)
    act, gu = B.k_gemm_swiglu(x, w)
    act_only, _ = B.k_gemm_swiglu(x, w, want_gate_up=False)             # the forward-only (teacher) form
    assert torch.equal(act, act_only)
    rows = sample_rows(M)
    up = round_bf16(f64(x[torch.as_tensor(rows, device="cuda")]) @ f64(w).T)
    _check_rows(gu, up, rows, TOL_BF16, name + " gate|up")
    _check_rows(act, round_bf16(ops.swiglu_fwd(up)), rows, TOL_BF16, name + " act")


# the two KD epilogues (statistics in pass 1, dz in pass 2) on a [16384, 8192] chunk with c2's hidden sizes, and on
# c5's hidden sizes with a ragged 4480-wide tail chunk behind a full one
KD_CASES = [("c2 chunk", 16384, 8192, 2048, 1024, 8192, 2.0), ("c5 hidden sizes, tail chunk", 8192, 8192 + 4480, 4096, 1536, 8192, 1.0)]


@pytest.mark.parametrize("name,n,V,Ht,Hs,Cv,T", KD_CASES, ids=[c[0] for c in KD_CASES])
def test_kd_epilogues_at_full_chunk_shape(name, n, V, Ht, Hs, Cv, T):
    kd = wl.KDConfig(V, Ht, Hs, T, Cv)
    h_t, h_s = dev("kht" + name, (n, Ht)), dev("khs" + name, (n, Hs))
    wt, ws = dev("kwt" + name, (V, Ht), 0.02), dev("kws" + name, (V, Hs), 0.02)
    d_ws = torch.zeros((V, Hs), dtype=torch.float32, device="cuda")
    out = B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws)
    ref = oracle_kd(f64(h_t), f64(h_s), f64(wt), f64(ws), T, 1.0 / n, round_bf16, token_block=2048)
    assert abs(out["loss"].item() - ref["loss"]) <= TOL_LOSS_BF16 * ref["loss"]
    assert_kl_tok(out["kl_tok"], ref["kl_tok"], TOL_LOSS_BF16, V)
    print("d_h_s", assert_parity(out["d_h_s"], ref["d_h_s"], TOL_BF16, "d_h_s"))
    print("d_w_s", assert_parity(d_ws, ref["d_w_s"], TOL_BF16, "d_w_s"))
