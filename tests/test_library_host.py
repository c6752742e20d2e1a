"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, the host
packing step matches the oracle, and argument errors are reported before anything is launched."""
import ctypes as C
import os
import re

import pytest

from oracle.packing import pack_microbatches as oracle_pack
from paper_2605_10501_amd import binding as B
from paper_2605_10501_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ms_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    syms = declared_symbols()
    assert "ms_section_forward" in syms and "ms_kd_loss_forward_backward" in syms and len(syms) >= 20
    for s in syms:
        assert hasattr(lib, s), s


@pytest.mark.parametrize("lengths,budget,policy", [
    ([5, 0, 3, 0, 4], 8, 0), ([2, 9, 2, 20, 9], 10, 1), ([0, 0], 16, 0), ([], 4, 1),
    ([7, 0, 1, 12, 5, 5, 0, 9], 16, 1), (wl.workload("c4").lengths, 32768, 0), (wl.workload("c4").lengths, 32768, 1)])
def test_pack_microbatches_matches_oracle(lengths, budget, policy):
    assert B.pack_microbatches(lengths, budget, policy) == tuple(oracle_pack(lengths, budget, policy))


def test_pack_rejects_bad_arguments():
    with pytest.raises(RuntimeError, match="token_budget"):
        B.pack_microbatches([1, 2], 0, 0)
    with pytest.raises(RuntimeError, match="negative"):
        B.pack_microbatches([1, -2], 8, 0)


def _call_forward(cfg_over=None, cu=(0, 4), n_tokens=4):
    cfg = wl.scaled(wl.workload("c1").student, **(cfg_over or {}))
    c = B._cfg_c(cfg)
    host = (C.c_int32 * len(cu))(*cu)
    b = B.BatchC(n_tokens, len(cu) - 1, C.c_void_p(256), host)
    layers = (B.LayerPtrs * cfg.n_layers)()
    for f in B._LAYER_FIELDS:
        setattr(layers[0], f, 256)
    w = B.SectionPtrs(256, layers, 256, 256)
    return B.lib().ms_section_forward(C.byref(c), C.byref(w), C.byref(b), C.c_void_p(256), C.c_void_p(256),
                                      C.c_void_p(256), C.c_size_t(16), None)


def test_errors_are_detected_on_the_host_without_a_gpu():
    assert _call_forward({"head_dim": 96}) == -4 and b"head_dim" in B.lib().ms_last_error()
    assert _call_forward({"n_q_heads": 3, "n_kv_heads": 2}) == -2
    assert _call_forward(cu=(0, 3, 2, 4)) == -1 and b"decreases" in B.lib().ms_last_error()
    assert _call_forward(cu=(0, 5), n_tokens=4) == -1
    assert _call_forward() == -3 and b"workspace" in B.lib().ms_last_error()      # 16-byte workspace
    assert _call_forward(cu=(0, 0), n_tokens=0) == 0                              # skipped section: no-op


def test_probe_arguments_are_checked_before_any_launch():
    lib = B.lib()
    assert lib.ms_k_clock_monitor(0, C.c_void_p(256), None) == -1
    assert lib.ms_k_clock_monitor(2_000_000, C.c_void_p(256), None) == -1        # longer than a second
    assert lib.ms_k_clock_monitor(100, None, None) == -1 and b"clock_monitor" in lib.ms_last_error()
    assert lib.ms_k_gemm_config(64, -1) == -1 and lib.ms_k_gemm_config(0, 2) == -1 and b"gemm_config" in lib.ms_last_error()
    assert lib.ms_k_gemm_config(256, 1) == 0 and lib.ms_k_gemm_config(0, -1) == 0
    assert lib.ms_k_mfma_probe(0, 10, 0, 0, C.c_void_p(256), None) == -1
    assert lib.ms_k_mfma_probe(4, 10, 1, 1, None, None) == -1


def test_workspace_sizes():
    c2 = wl.workload("c2")
    fwd = B.section_workspace_bytes(c2.teacher, 16384, 4096, False)
    bwd = B.section_workspace_bytes(c2.student, 16384, 4096, True)
    assert 0 < fwd < 4 << 30 and 0 < bwd < 8 << 30
    assert B.section_workspace_bytes(wl.scaled(c2.student, head_dim=100), 16, 16, True) == 0
    kd = B.kd_workspace_bytes(wl.workload("c3").kd, 8192)
    assert kd >= 2 * 8192 * 8192 * 4 and kd < 2 << 30


def test_static_scratch_kd_call_rejects_oversize_before_touching_the_device():
    kd = wl.KDConfig(151936, 4096, 2048, 2.0, 8192)
    c = B.KDConfigC(kd.vocab, kd.h_teacher, kd.h_student, kd.chunk, B.MS_BF16, kd.temperature, 1.0, 256, 256, 0)
    fake = C.c_void_p(256)
    assert B.kd_workspace_bytes(kd, 8192) > B.KD_STATIC_SCRATCH_BYTES
    assert B.lib().ms_kd_loss_forward_backward_static(C.byref(c), 8192, fake, fake, fake, fake, fake, fake, None) == -3
    assert b"built-in buffer" in B.lib().ms_last_error()
