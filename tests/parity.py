"""Parity metric between the HIP path and the oracle.

err_i = |gpu_i - ref_i| / max(|ref_i|, rms(ref)); every element must be within the tolerance.
The rms floor makes the relative error meaningful for elements near zero.
"""
import numpy as np
import torch

TOL_BF16 = 2e-2      # bf16 activations and gradients
TOL_F32 = 1e-4       # fp32 runs; also fp32 results computed from bf16 inputs
TOL_LOSS_BF16 = 1e-3
TOL_LOSS_F32 = 1e-4


def rel_err(gpu, ref):
    g = gpu.detach().to(torch.float64).cpu().numpy() if isinstance(gpu, torch.Tensor) else np.asarray(gpu, np.float64)
    r = np.asarray(ref, dtype=np.float64).reshape(g.shape)
    rms = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
    den = np.maximum(np.abs(r), max(rms, 1e-300))
    return np.abs(g - r) / den


def assert_parity(gpu, ref, tol, name=""):
    e = rel_err(gpu, ref)
    assert np.all(np.isfinite(e)), f"{name}: non-finite values"
    mx = float(e.max()) if e.size else 0.0
    assert mx <= tol, f"{name}: max err {mx:.3e} > {tol:.1e} (p99.9 {np.quantile(e, 0.999):.3e}, at {np.unravel_index(e.argmax(), e.shape)})"
    return mx
