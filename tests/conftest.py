import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


# Kernel selections of the bf16 GEMMs that the shapes of the tests would not all reach by themselves: the
# automatic choice, both workgroup tiles with both MFMA shapes, and the generic kernel.
GEMM_CONFIGS = [(0, -1), (256, 1), (256, 0), (128, 1), (128, 0), (-1, -1)]


@pytest.fixture(params=GEMM_CONFIGS, ids=lambda c: f"tile{c[0]}_mfma{c[1]}")
def gemm_config(request):
    from paper_2605_10501_amd import binding as B
    B.k_gemm_config(*request.param)
    yield request.param
    B.k_gemm_config(0, -1)


@pytest.fixture
def rng():
    return np.random.default_rng(1234)


def fd_grad(f, x, idx, h=1e-6):
    """Central finite difference of scalar f with respect to x[idx] (x float64, modified in place and restored)."""
    old = x[idx]
    x[idx] = old + h
    fp = f()
    x[idx] = old - h
    fm = f()
    x[idx] = old
    return (fp - fm) / (2 * h)
