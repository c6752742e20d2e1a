"""Host-side checks of the synthetic workload generator (no method arithmetic in it)."""
import os

import numpy as np
import torch

from paper_2605_10501_amd import workloads as wl
from oracle.packing import pack_microbatches

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_counter_generator_is_a_pure_function_of_seed_tag_index():
    a = wl.normal(0, "x", (1000,), chunk=128)
    b = wl.normal(0, "x", (1000,))
    assert torch.equal(a, b)                                                    # chunking invisible
    assert torch.equal(wl.normal(0, "x", (10,)), b[:10])                        # element i independent of n
    assert not torch.equal(wl.normal(1, "x", (1000,)), b) and not torch.equal(wl.normal(0, "y", (1000,)), b)


def test_normal_and_uniform_moments():
    z = wl.normal(3, "m", (1 << 18,), std=0.02, mean=1.0).double()
    assert abs(z.mean().item() - 1.0) < 2e-4 and abs(z.std().item() - 0.02) < 2e-4
    u = wl.uniform(3, "u", 1 << 18).double()
    assert 0 < u.min().item() and u.max().item() < 1 and abs(u.mean().item() - 0.5) < 3e-3
    r = wl.randint(3, "r", 1 << 16, 16, 129)
    assert r.min().item() == 16 and r.max().item() == 128


def test_workload_shapes_follow_the_configs():
    c1 = wl.workload("c1")
    assert len(c1.lengths) == 4 and all(16 <= n <= 128 for n in c1.lengths) and c1.n_tokens == sum(c1.lengths)
    c2 = wl.workload("c2")
    assert sum(c2.lengths) == 16384 and max(c2.lengths) <= 4096 and all(n >= 64 for n in c2.lengths[:-1])
    assert c2.teacher.d_qkv == 3072 and c2.student.d_up == 5632 and c2.teacher.layer_params() == 44302336
    c4 = wl.workload("c4")
    assert len(c4.lengths) == 64 and sum(1 for n in c4.lengths if n == 0) == 19
    assert all(256 <= n <= 4096 for n in c4.lengths if n)
    c5 = wl.workload("c5")
    assert sum(c5.lengths) == 32768 and c5.student.layer_params() == 46792704


def test_text_only_samples_skip_the_encoder_section():
    c4 = wl.workload("c4")
    order, off, cus = pack_microbatches(c4.lengths, 1 << 30, 0)
    assert len(order) == 45 and all(c4.lengths[i] > 0 for i in order)
    assert cus[0] == wl.cu_seqlens_of(c4.lengths)


def test_weights_recipe():
    cfg = wl.scaled(wl.workload("c4").student, n_layers=1)
    w = wl.section_weights(cfg, 0, "vit")
    lw = w["layers"][0]
    assert lw["w_qkv"].shape == (3840, 1280) and lw["b_up"].shape == (5120,) and lw["w_up"].dtype == torch.bfloat16
    assert abs(lw["norm1_g"].float().mean().item() - 1.0) < 5e-3 and abs(lw["w_down"].float().std().item() - 0.02) < 1e-3
    f = wl.to_f64(w)
    assert f["layers"][0]["w_o"].dtype == np.float64 and "embedding" not in f


def test_logits_to_hidden_ratio_printed_in_the_paper():
    for line in open(os.path.join(GOLDEN, "logits_vs_hidden.txt")):
        if line.startswith("#"):
            continue
        v, h, ratio = line.split()
        assert int(v) / int(h) == float(ratio)
    kd = wl.workload("c3").kd
    assert round(kd.vocab / kd.h_teacher, 1) == 37.1
