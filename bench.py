#!/usr/bin/env python3
"""One-GPU benchmark of the section hot path on the mid-size distillation workload (c2).

A step = one packed micro-batch of 16384 tokens through the whole path: teacher section forward
(8 layers), student section forward + KD loss + backward (4 layers).  Prints ONE JSON line:
whole-step tokens/s, the roofline of the dominant kernel (bf16 MFMA GEMM) from per-launch HIP
events recorded by the library, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def model_flops(work):
    """Algorithmic flops of one step: GEMMs 2*M*N*K, causal attention over unmasked pairs only,
    backward = 2x GEMM forward and 2.5x attention forward, KD without the pass-2 recompute."""
    n = work.n_tokens
    pairs = sum(l * (l + 1) // 2 for l in work.lengths if l)

    def section(cfg, bwd):
        gemm = 2.0 * cfg.layer_params() * n * cfg.n_layers
        attn = 4.0 * cfg.n_q_heads * cfg.head_dim * pairs * cfg.n_layers
        return (gemm * 3 + attn * 3.5) if bwd else (gemm + attn)

    kd = work.kd
    return dict(teacher=section(work.teacher, False), student=section(work.student, True),
                kd=2.0 * n * kd.vocab * (kd.h_teacher + kd.h_student) + 4.0 * n * kd.vocab * kd.h_student)


def _tensors(tree):
    """All tensors of a nested dict / list of weights."""
    if isinstance(tree, dict):
        for v in tree.values():
            yield from _tensors(v)
    elif isinstance(tree, (list, tuple)):
        for v in tree:
            yield from _tensors(v)
    elif tree is not None and hasattr(tree, "numel"):
        yield tree


def describe(c):
    return f"{c.n_layers}L d{c.d_model} {c.n_q_heads}/{c.n_kv_heads} heads hd{c.head_dim} F{c.d_ffn}"


def nt_gemm_shapes(work):
    """(M, N, K, bytes written per output element, bytes read per output element besides A and B) of every
    A[M,K]*B[N,K]^T launch of one step (decoder sections, bf16 fast path with its fused epilogues)."""
    n = work.n_tokens
    out = []
    for cfg, bwd in ((work.teacher, False), (work.student, True)):
        d, f = cfg.d_model, cfg.d_ffn
        qkv = (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim
        # gate/up + SwiGLU: N = 2F accumulator columns; writes act [n, F] (1 B per accumulator column) and, when a
        # backward pass follows, the pre-activations [n, 2F] as well
        per_layer = [(n, qkv, d, 2, 0), (n, d, cfg.n_q_heads * cfg.head_dim, 4, 4), (n, 2 * f, d, 3 if bwd else 1, 0),
                     (n, d, f, 4, 4)]
        out += per_layer * cfg.n_layers
    kd = work.kd
    for v0 in range(0, kd.vocab, kd.chunk):
        cw = min(kd.chunk, kd.vocab - v0)
        # teacher logits stored fp32 in both passes; student logits consumed by their epilogue together with the
        # teacher's (statistics: nothing but 0.5 B of partials per column; dz: 2 B)
        out += [(n, cw, kd.h_teacher, 4, 0), (n, cw, kd.h_student, 0.5, 4), (n, cw, kd.h_teacher, 4, 0), (n, cw, kd.h_student, 2, 4)]
    return out


def measured_traffic():
    """HBM-side bytes per NT launch from the committed counter summary (two rocprofv3 --pmc runs), or None."""
    path = os.path.join(ROOT, "profiles", "gemm_bf16_fast_kernel_c2_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("gemm_nt_traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--step-only", action="store_true",
                    help="skip the side measurements (teacher sweep, AdamW, references): for profiler runs of the step")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run the library's copy kernel 3x on MIB MiB (reference dispatch for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's section compute; this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_10501_amd import binding as B
    from paper_2605_10501_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = "cuda"
    work = wl.workload(args.workload, 0)
    if work.teacher is None:     # c3 (KD head alone) and c4 (vision encoder forward+backward): secondary workloads
        print(json.dumps(bench_secondary(work, args, torch, B, wl, dev)))
        return
    t_cfg, s_cfg, kd = work.teacher, work.student, work.kd
    dt = t_cfg.torch_dtype
    tw, sw = wl.section_weights(t_cfg, 0, "teacher", dev), wl.section_weights(s_cfg, 0, "student", dev)
    wt = wl.normal(0, "lm_head.t", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, dev)
    ws = wl.normal(0, "lm_head.s", (kd.vocab, kd.h_student), 0.02, 0.0, dt, dev)
    cu = wl.cu_seqlens_of(work.lengths)
    n = cu[-1]
    ids = wl.randint(0, "ids", n, 0, t_cfg.vocab, dev)
    batch = B.Batch(cu)
    grads = B.zero_grads(sw)
    d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device=dev)
    ws_t = B.workspace(B.section_workspace_bytes(t_cfg, n, batch.max_seqlen, False), dev, "teacher")
    ws_s = B.workspace(B.section_workspace_bytes(s_cfg, n, batch.max_seqlen, True) + B.kd_workspace_bytes(kd, n), dev, "student")
    h_t = torch.empty((n, t_cfg.d_model), dtype=dt, device=dev)

    def teacher():
        return B.section_forward(t_cfg, tw, batch, ids, h_out=h_t, ws=ws_t)

    def student():
        return B.section_forward_backward(s_cfg, sw, grads, batch, ids, kd=kd, w_teacher=wt, w_student=ws,
                                          h_teacher=h_t, d_w_student=d_ws, ws=ws_s)

    def step():
        teacher()
        return student()

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            out = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k, out

    if args.copy_calibration:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            B.k_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    sec_step, out = timed(step, args.steps)
    loss = float(out["loss"].item())
    sec_teacher, _ = timed(teacher, args.steps)
    sec_student, _ = timed(student, args.steps)
    # the KD head alone (both lm_heads, loss, gradients to the student hidden states and lm_head) on this batch
    sec_kd = float("nan")
    if not args.step_only:
        h_s = wl.normal(0, "bench.h_s", (n, kd.h_student), 1.0, 0.0, dt, dev)
        sec_kd, _ = timed(lambda: B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws), args.steps)

    # per-kernel durations from HIP events on the launch stream (separate, untimed-for-value steps)
    B.profile_enable(1)
    prof_steps = min(args.steps, 3)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = B.profile_read()
    B.profile_enable(0)
    sweep, adamw, probe_tflops, probe_rand_tflops, probe16_rand_tflops, copy_gbs, variant = [], None, None, None, None, None, None
    clocks = {}
    side = torch.cuda.Stream()
    clk = torch.zeros(2, dtype=torch.int64, device=dev)

    def clock_during(fn, reps, microseconds):
        """Average shader clock (MHz) while `reps` x fn run: fn is queued on the main stream, then one wave on a
        second stream compares the shader-clock counter with the constant 100 MHz counter for `microseconds`."""
        torch.cuda.synchronize()
        for _ in range(reps):
            fn()
        with torch.cuda.stream(side):
            B.k_clock_monitor(microseconds, clk)
        torch.cuda.synchronize()
        c, w = clk.tolist()
        return 100.0 * c / max(w, 1)

    if not args.step_only:
        # variant (not the metric): a token block's teacher logits stay in HBM between the two KD passes instead
        # of being recomputed -- [4096, vocab] fp32, independent of the batch size
        kd_v = wl.scaled(kd, token_block=4096)
        ws_v = B.workspace(B.section_workspace_bytes(s_cfg, n, batch.max_seqlen, True) + B.kd_workspace_bytes(kd_v, n), dev, "variant")

        def step_v():
            teacher()
            return B.section_forward_backward(s_cfg, sw, grads, batch, ids, kd=kd_v, w_teacher=wt, w_student=ws,
                                              h_teacher=h_t, d_w_student=d_ws, ws=ws_v)
        step_v()
        sec_v, out_v = timed(step_v, args.steps)
        variant = {"kd_token_block": 4096, "tokens_per_s": n / sec_v, "ms_per_step": 1e3 * sec_v,
                   "teacher_logits_cache_bytes": 4096 * kd.vocab * 4, "loss": float(out_v["loss"].item())}
        # teacher micro-batch sweep (Sec. 4.2: a forward-only teacher is under-utilised by small micro-batches):
        # forward rate and workspace of the teacher section at 1, 2, 4, 8 packed samples of 4096 tokens
        sweep = []
        for k in (1, 2, 4, 8):
            nt = 4096 * k
            bt = B.Batch([4096 * i for i in range(k + 1)])
            ids_k = wl.randint(0, "sweep.ids", nt, 0, t_cfg.vocab, dev)
            need = B.section_workspace_bytes(t_cfg, nt, 4096, False)
            wsk = B.workspace(need, dev, "sweep")
            sec_k, _ = timed(lambda: B.section_forward(t_cfg, tw, bt, ids_k, ws=wsk), max(3, args.steps // 2))
            sweep.append({"samples": k, "tokens": nt, "tokens_per_s": nt / sec_k, "workspace_bytes": need})
        # the student's AdamW update over all its parameters (outside the timed step: the metric is the KD step)
        n_par = sum(t.numel() for t in _tensors(sw)) + ws.numel()
        n_par -= n_par % 4
        st = [torch.zeros(n_par, dtype=torch.float32, device=dev) for _ in range(4)]
        w_model = torch.empty(n_par, dtype=dt, device=dev)
        sec_opt, _ = timed(lambda: B.adamw_step(st[0], st[1], st[2], st[3], w_model, 1, lr=1e-4, weight_decay=0.1), 5)
        adamw = {"parameters": n_par, "ms": 1e3 * sec_opt, "GB/s": n_par * 30.0 / sec_opt / 1e9}
        del st, w_model
        # what the chip sustains on this machine: register-resident MFMA loop and a plain 1 GiB copy (references beside
        # the published peaks)
        sink = torch.zeros(512 * 512, dtype=torch.float32, device=dev)
        sec_probe, _ = timed(lambda: B.k_mfma_probe(512, 10000, sink), 3)
        probe_tflops = 512 * 8 * 10000 * 8 * 32768 / sec_probe / 1e12
        # the same loop on operands with random signs and mantissas: the chip lowers its clock under their bit
        # activity, so this is the rate a bf16 kernel can approach on real data
        sec_probe_r, _ = timed(lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True), 3)
        probe_rand_tflops = 512 * 8 * 10000 * 8 * 32768 / sec_probe_r / 1e12
        clocks["mfma_register_loop"] = clock_during(lambda: B.k_mfma_probe(512, 10000, sink), 4, int(3e6 * sec_probe))
        clocks["mfma_register_loop_random_operands"] = clock_during(
            lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True), 4, int(3e6 * sec_probe_r))
        # the 16x16x32 shape the GEMMs use, on random operands
        sec_probe_16, _ = timed(lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True, mfma16=True), 3)
        probe16_rand_tflops = 512 * 8 * 10000 * 8 * 32768 / sec_probe_16 / 1e12
        clocks["mfma16_register_loop_random_operands"] = clock_during(
            lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True, mfma16=True), 4, int(3e6 * sec_probe_16))
        clocks["whole_step"] = clock_during(step, 3, int(2e6 * sec_step))
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        sec_copy, _ = timed(lambda: B.k_copy(src, dst), 3)
        copy_gbs = 2.0 * (1 << 30) / sec_copy / 1e9
        del src, dst, sink
    fl = model_flops(work)
    g_n, g_ms, g_work = prof["gemm_nt"]
    gt_n, gt_ms, gt_work = prof["gemm_t"]
    achieved = g_work / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    kernels = {}
    for name, (cnt, ms, workv) in prof.items():
        if cnt:
            kernels[name] = {"launches_per_step": cnt / prof_steps, "ms_per_step": ms / prof_steps,
                             "avg_us": 1e3 * ms / cnt}
            if workv > 0:
                unit = "TFLOP/s" if name.startswith("gemm") else "GB/s"
                kernels[name][unit] = workv / (ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
    total_flops = fl["teacher"] + fl["student"] + fl["kd"]
    alg_bytes = traffic = None
    if work.teacher.arch == "decoder" and work.student.arch == "decoder":
        shapes = nt_gemm_shapes(work)
        if len(shapes) == g_n / prof_steps and abs(sum(2.0 * m * nn * k for m, nn, k, _, _ in shapes) * prof_steps / g_work - 1) < 1e-3:
            alg_bytes = sum(2.0 * (m * k + nn * k) + (ob + rb) * m * nn for m, nn, k, ob, rb in shapes) / len(shapes)
        if args.workload == "c2":
            traffic = measured_traffic()
    result = {
        "metric": "KD step tokens/s (teacher fwd + student fwd+bwd + fused KL loss), 1 GPU",
        "value": n / sec_step, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * sec_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{work.name}: KD step, {n} packed tokens, {batch.n_seqs} sequences (max {batch.max_seqlen}), "
                               f"teacher {describe(t_cfg)}, student {describe(s_cfg)}, vocab {kd.vocab}, "
                               f"T={kd.temperature:g}, chunk {kd.chunk}"},
        "teacher_fwd_tokens_per_s": n / sec_teacher, "student_fwd_bwd_kd_tokens_per_s": n / sec_student,
        "kd_loss_fwd_bwd_tokens_per_s": None if args.step_only else n / sec_kd,
        "mfma_frac_kd_loss": None if args.step_only else fl["kd"] / sec_kd / 1e12 / PEAK_BF16_TFLOPS,
        "model_tflop_per_step": total_flops / 1e12,
        "mfma_frac_whole_step": total_flops / sec_step / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_frac_teacher_fwd": fl["teacher"] / sec_teacher / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_frac_student_fwd_bwd_kd": (fl["student"] + fl["kd"]) / sec_student / 1e12 / PEAK_BF16_TFLOPS,
        "loss": loss, "logits_to_hidden_ratio": kd.vocab / kd.h_teacher,
        "variant_cached_teacher_logits": variant, "teacher_microbatch_sweep": sweep, "student_adamw_step": adamw,
        "measured_references": None if args.step_only else {"mfma_register_loop_tflops": probe_tflops,
                                                             "mfma_register_loop_random_operands_tflops": probe_rand_tflops,
                                                             "mfma16_register_loop_random_operands_tflops": probe16_rand_tflops,
                                                             "shader_clock_mhz": clocks,
                                                             "copy_1gib_read_plus_write_gbs": copy_gbs},
        "roofline": {"kernel": "gemm_bf16_fast_kernel (A[M,K] B[N,K]^T, all forward linears and lm_head chunks)",
                     "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": "profiles/gemm_bf16_fast_kernel_c2_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE, "
                                       "WRITE_SIZE; bytes per launch)" if traffic else None,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "launches_per_step": g_n / prof_steps, "avg_launch_us": 1e3 * g_ms / max(g_n, 1),
                     "flops_per_launch_avg": g_work / max(g_n, 1)},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(work, tw, sw, wt, ws, ids, args.cpu_sample_tokens)
    print(json.dumps(result))


def bench_secondary(work, args, torch, B, wl, dev):
    """c3: the KD head alone on given hidden states; c4: one vision-encoder section forward+backward on a packed
    micro-batch of image samples.  Same timing protocol as the main step; no roofline object (not the metric's workload)."""
    dt = torch.bfloat16

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k
    if work.student is None:
        kd, n = work.kd, work.n_tokens
        h_t = wl.normal(0, "c3.ht", (n, kd.h_teacher), 1.0, 0.0, dt, dev)
        h_s = wl.normal(0, "c3.hs", (n, kd.h_student), 1.0, 0.0, dt, dev)
        wt = wl.normal(0, "c3.wt", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, dev)
        ws = wl.normal(0, "c3.ws", (kd.vocab, kd.h_student), 0.02, 0.0, dt, dev)
        d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device=dev)
        wsb = B.workspace(B.kd_workspace_bytes(kd, n), dev, "kd")
        fn = lambda: B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws, ws=wsb)
        flops = 2.0 * n * kd.vocab * (kd.h_teacher + kd.h_student) + 4.0 * n * kd.vocab * kd.h_student
        metric = "KD head tokens/s (both lm_heads, KL loss, gradients to student hidden states and lm_head), 1 GPU"
        desc = f"{work.name}: {n} tokens, vocab {kd.vocab} in chunks of {kd.chunk}, hidden {kd.h_teacher}/{kd.h_student}, T={kd.temperature:g}"
    else:
        cfg = work.student
        cu = wl.cu_seqlens_of(work.lengths)
        n, batch = cu[-1], B.Batch(cu)
        w = wl.section_weights(cfg, 0, "vit", dev)
        grads = B.zero_grads(w)
        x = wl.normal(0, "c4.x", (n, cfg.d_model), 1.0, 0.0, dt, dev)
        dy = wl.normal(0, "c4.dy", (n, cfg.d_model), 1.0, 0.0, dt, dev)
        wsb = B.workspace(B.section_workspace_bytes(cfg, n, batch.max_seqlen, True), dev, "vit")
        fn = lambda: B.section_forward_backward(cfg, w, grads, batch, x, d_h_out=dy, ws=wsb)
        pairs = sum(l * l for l in work.lengths if l)
        flops = 3 * 2.0 * cfg.layer_params() * n * cfg.n_layers + 3.5 * 4.0 * cfg.n_q_heads * cfg.head_dim * pairs * cfg.n_layers
        metric = "vision-encoder section forward+backward tokens/s, 1 GPU"
        desc = f"{work.name}: {n} packed patch tokens, {batch.n_seqs} image samples (max {batch.max_seqlen}), {describe(cfg)}, bidirectional"
    for _ in range(args.warmup):
        fn()
    sec = timed(fn, args.steps)
    B.profile_enable(1)
    fn()
    torch.cuda.synchronize()
    prof = B.profile_read()
    B.profile_enable(0)
    kernels = {k: {"launches": c, "ms": ms} for k, (c, ms, _) in prof.items() if c}
    return {"metric": metric, "value": n / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": 1e3 * sec, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
            "data": "synthetic", "config": {"workload": desc}, "model_tflop_per_step": flops / 1e12,
            "mfma_frac_whole_step": flops / sec / 1e12 / PEAK_BF16_TFLOPS, "kernels": kernels}


def cpu_baseline(work, tw, sw, wt, ws, ids, sample_tokens):
    """The oracle as it stands, timed on the first `sample_tokens` tokens of the same batch
    (sequences truncated to fit), all host threads numpy's BLAS uses."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import round_bf16, round_f32
    from oracle.section import SectionSpec
    from oracle.step import distill_step
    from paper_2605_10501_amd import workloads as wl

    def spec(c):
        return SectionSpec(c.arch, c.n_layers, c.d_model, c.n_q_heads, c.n_kv_heads, c.head_dim, c.d_ffn, c.vocab,
                           c.norm_eps, c.rope_base)
    lens, tot = [], 0
    for l in work.lengths:
        if l and tot < sample_tokens:
            lens.append(min(l, sample_tokens - tot))
            tot += lens[-1]
    cu = wl.cu_seqlens_of(lens)
    t_w, s_w, w_t, w_s = wl.to_f64(tw), wl.to_f64(sw), wl.to_f64(wt), wl.to_f64(ws)
    ids_h = ids[:tot].cpu().numpy()
    t0 = time.perf_counter()
    out = distill_step(spec(work.teacher), t_w, spec(work.student), s_w, cu, ids_h, w_t, w_s,
                       work.kd.temperature, 1.0 / tot, round_bf16, rnd_res=round_f32)
    sec = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": tot / sec, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {tot} tokens of the same batch ({len(lens)} sequences), full model widths and vocab, "
                      f"{sec:.1f} s of fp64 numpy work", "loss": out["loss"]}


if __name__ == "__main__":
    main()
