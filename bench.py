#!/usr/bin/env python3
"""One-GPU benchmark of the section hot path.

Headline (`value`): the largest single-GPU workload, c5 -- one packed micro-batch of 32768 tokens through the whole
path: teacher section forward (4 layers, d 4096), student section forward + fused KD loss + backward (4 layers,
d 1536, vocab 151936).  The same JSON line carries the other workloads as sub-objects (`workloads`: c2 = the mid-size
KD step, c3 = the large-vocabulary KD head alone, c4 = the vision-encoder section forward+backward), each timed with
the same protocol, the roofline of the dominant kernel (bf16 MFMA GEMM) from per-launch HIP events recorded by the
library on the launch stream, per-kernel-class rates against the MFMA / HBM peaks, and the CPU oracle timed on a
bounded sample of the headline workload.  `--workload c2|c3|c4|c5` runs one workload alone (profiler runs).
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
MFMA_CLASSES = ("gemm_nt", "gemm_t", "attn_fwd", "attn_bwd")


def section_flops(cfg, n, pairs, bwd):
    """Algorithmic flops of a section: GEMMs 2*M*N*K, attention 4*nq*hd per (query, visible key) pair; backward =
    2x GEMM forward and 2.5x attention forward."""
    gemm = 2.0 * cfg.layer_params() * n * cfg.n_layers
    attn = 4.0 * cfg.n_q_heads * cfg.head_dim * pairs * cfg.n_layers
    return (gemm * 3 + attn * 3.5) if bwd else (gemm + attn)


def kd_flops(kd, n):
    """Without the pass-2 recompute of the logits."""
    return 2.0 * n * kd.vocab * (kd.h_teacher + kd.h_student) + 4.0 * n * kd.vocab * kd.h_student


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
    A[M,K]*B[N,K]^T launch of one KD step (decoder sections, bf16 fast path with its fused epilogues)."""
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


def measured_traffic(name):
    """HBM-side bytes per NT-GEMM launch from the committed counter summary (two rocprofv3 --pmc runs), or None."""
    path = os.path.join(ROOT, "profiles", f"gemm_bf16_fast_kernel_{name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("gemm_nt_traffic_bytes_per_launch:"):
                return float(line.split(":")[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def timed(torch, fn, k):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = None
    for _ in range(k):
        out = fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / k, out


def kernel_table(prof, prof_steps, attn_flops):
    """Per kernel class: launches and time per step, achieved rate, fraction of the peak that bounds the class
    (bf16 MFMA for GEMM / attention, HBM for everything else).  attn_flops = (forward, backward) algorithmic flops of
    one step's attention launches (the library cannot know the sequence lengths' pair count per launch)."""
    kernels = {}
    for name, (cnt, ms, workv) in prof.items():
        if not cnt:
            continue
        k = {"launches_per_step": cnt / prof_steps, "ms_per_step": ms / prof_steps, "avg_us": 1e3 * ms / cnt}
        if name == "attn_fwd":
            workv = attn_flops[0] * prof_steps
        elif name == "attn_bwd":
            workv = attn_flops[1] * prof_steps
        if workv > 0 and ms > 0:
            if name in MFMA_CLASSES:
                k["TFLOP/s"] = workv / (ms * 1e-3) / 1e12
                k["frac_of_mfma_peak"] = k["TFLOP/s"] / PEAK_BF16_TFLOPS
            else:
                k["GB/s"] = workv / (ms * 1e-3) / 1e9
                k["frac_of_hbm_peak"] = k["GB/s"] / PEAK_HBM_GBS
        kernels[name] = k
    return kernels


def progress(args, what):
    """One line on stderr per phase in --dispatch-only mode, so that a profiler run that stops shows where."""
    if getattr(args, "dispatch_only", False):
        print(f"[bench] {what}", file=sys.stderr, flush=True)


def profile_steps(torch, B, fn, steps):
    B.profile_enable(1)
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    prof = B.profile_read()
    B.profile_enable(0)
    return prof


def bench_kd_step(name, args, torch, B, wl, dev, side):
    """c2 / c5: teacher forward + student forward + KD loss + backward on one packed micro-batch."""
    work = wl.workload(name, 0)
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

    if args.copy_calibration:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            B.k_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst
    progress(args, f"{name}: inputs and weights resident, first launch next")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    progress(args, f"{name}: warm-up done")
    sec_step, out = timed(torch, step, args.steps)
    loss = float(out["loss"].item())
    progress(args, f"{name}: timed steps done")
    if args.dispatch_only:
        return {"workload": work.name, "n_tokens": n, "ms_per_step": 1e3 * sec_step, "loss": loss}
    sec_teacher, _ = timed(torch, teacher, args.steps)
    sec_student, _ = timed(torch, student, args.steps)
    sec_kd = None
    if not args.step_only:
        # the KD head alone (both lm_heads, loss, gradients to the student hidden states and lm_head) on this batch
        h_s = wl.normal(0, "bench.h_s", (n, kd.h_student), 1.0, 0.0, dt, dev)
        sec_kd, _ = timed(torch, lambda: B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws), max(2, args.steps // 2))
        del h_s
    prof_steps = min(args.steps, 3)
    prof = profile_steps(torch, B, step, prof_steps)

    pairs = sum(l * (l + 1) // 2 for l in work.lengths if l)
    fl = dict(teacher=section_flops(t_cfg, n, pairs, False), student=section_flops(s_cfg, n, pairs, True), kd=kd_flops(kd, n))
    att = lambda c: 4.0 * c.n_q_heads * c.head_dim * pairs * c.n_layers
    kernels = kernel_table(prof, prof_steps, (att(t_cfg) + att(s_cfg), 2.5 * att(s_cfg)))
    g_n, g_ms, g_work = prof["gemm_nt"]
    achieved = g_work / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    alg_bytes = None
    shapes = nt_gemm_shapes(work)
    if len(shapes) == g_n / prof_steps and abs(sum(2.0 * m * nn * k for m, nn, k, _, _ in shapes) * prof_steps / g_work - 1) < 1e-3:
        alg_bytes = sum(2.0 * (m * k + nn * k) + (ob + rb) * m * nn for m, nn, k, ob, rb in shapes) / len(shapes)
    traffic, traffic_src = measured_traffic(name)
    total_flops = fl["teacher"] + fl["student"] + fl["kd"]
    res = {
        "workload": f"{work.name}: KD step, {n} packed tokens, {batch.n_seqs} sequences (max {batch.max_seqlen}), "
                    f"teacher {describe(t_cfg)}, student {describe(s_cfg)}, vocab {kd.vocab}, T={kd.temperature:g}, chunk {kd.chunk}",
        "n_tokens": n, "ms_per_step": 1e3 * sec_step, "tokens_per_s": n / sec_step,
        "teacher_fwd_tokens_per_s": n / sec_teacher, "student_fwd_bwd_kd_tokens_per_s": n / sec_student,
        "kd_loss_fwd_bwd_tokens_per_s": n / sec_kd if sec_kd else None,
        "model_tflop_per_step": total_flops / 1e12,
        "mfma_frac_whole_step": total_flops / sec_step / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_frac_teacher_fwd": fl["teacher"] / sec_teacher / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_frac_student_fwd_bwd_kd": (fl["student"] + fl["kd"]) / sec_student / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_frac_kd_loss": fl["kd"] / sec_kd / 1e12 / PEAK_BF16_TFLOPS if sec_kd else None,
        "student_section_tflops": (fl["student"] + fl["kd"]) / sec_student / 1e12,
        "loss": loss, "logits_to_hidden_ratio": kd.vocab / kd.h_teacher,
        "roofline": {"kernel": "gemm_bf16_fast_kernel (A[M,K] B[N,K]^T: all forward linears and lm_head chunk GEMMs)",
                     "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": (traffic_src + " (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; bytes per launch)") if traffic else None,
                     "algorithmic_bytes_per_launch": alg_bytes, "launches_per_step": g_n / prof_steps,
                     "avg_launch_us": 1e3 * g_ms / max(g_n, 1), "flops_per_launch_avg": g_work / max(g_n, 1)},
        "kernels": kernels,
    }
    if side and not args.step_only:
        res.update(side_measurements(args, torch, B, wl, dev, work, tw, sw, wt, ws, ids, batch, grads, d_ws, h_t, teacher, step, sec_step))
    if args.cpu_baseline_here:
        res["cpu_baseline"] = cpu_baseline(work, tw, sw, wt, ws, ids, args.cpu_sample_tokens)
    return res


def side_measurements(args, torch, B, wl, dev, work, tw, sw, wt, ws, ids, batch, grads, d_ws, h_t, teacher, step, sec_step):
    """Measurements beside the metric (c2 shapes): cached-teacher-logits variant, teacher micro-batch sweep, AdamW,
    the chip's sustained MFMA and copy rates and the shader clocks granted under load."""
    t_cfg, s_cfg, kd = work.teacher, work.student, work.kd
    n, dt = batch.n_tokens, t_cfg.torch_dtype
    side = torch.cuda.Stream()
    clk = torch.zeros(2, dtype=torch.int64, device=dev)
    clocks = {}

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

    # variant (not the metric): a token block's teacher logits stay in HBM between the two KD passes instead
    # of being recomputed -- [4096, vocab] fp32, independent of the batch size
    kd_v = wl.scaled(kd, token_block=4096)
    ws_v = B.workspace(B.section_workspace_bytes(s_cfg, n, batch.max_seqlen, True) + B.kd_workspace_bytes(kd_v, n), dev, "variant")

    def step_v():
        teacher()
        return B.section_forward_backward(s_cfg, sw, grads, batch, ids, kd=kd_v, w_teacher=wt, w_student=ws,
                                          h_teacher=h_t, d_w_student=d_ws, ws=ws_v)
    step_v()
    sec_v, out_v = timed(torch, step_v, args.steps)
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
        sec_k, _ = timed(torch, lambda: B.section_forward(t_cfg, tw, bt, ids_k, ws=wsk), max(3, args.steps // 2))
        sweep.append({"samples": k, "tokens": nt, "tokens_per_s": nt / sec_k, "workspace_bytes": need})
    # the student's AdamW update over all its parameters (outside the timed step: the metric is the KD step)
    n_par = sum(t.numel() for t in _tensors(sw)) + ws.numel()
    n_par -= n_par % 4
    st = [torch.zeros(n_par, dtype=torch.float32, device=dev) for _ in range(4)]
    w_model = torch.empty(n_par, dtype=dt, device=dev)
    sec_opt, _ = timed(torch, lambda: B.adamw_step(st[0], st[1], st[2], st[3], w_model, 1, lr=1e-4, weight_decay=0.1), 5)
    adamw = {"parameters": n_par, "ms": 1e3 * sec_opt, "GB/s": n_par * 30.0 / sec_opt / 1e9,
             "frac_of_hbm_peak": n_par * 30.0 / sec_opt / 1e9 / PEAK_HBM_GBS}
    del st, w_model
    # what the chip sustains on this machine: register-resident MFMA loop and a plain 1 GiB copy (references beside
    # the published peaks)
    sink = torch.zeros(512 * 512, dtype=torch.float32, device=dev)
    probe_flops = 512 * 8 * 10000 * 8 * 32768
    sec_probe, _ = timed(torch, lambda: B.k_mfma_probe(512, 10000, sink), 3)
    # the same loop on operands with random signs and mantissas: the chip lowers its clock under their bit
    # activity, so this is the rate a bf16 kernel can approach on real data
    sec_probe_r, _ = timed(torch, lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True), 3)
    clocks["mfma_register_loop"] = clock_during(lambda: B.k_mfma_probe(512, 10000, sink), 4, int(3e6 * sec_probe))
    clocks["mfma_register_loop_random_operands"] = clock_during(
        lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True), 4, int(3e6 * sec_probe_r))
    # the 16x16x32 shape the GEMMs use, on random operands
    sec_probe_16, _ = timed(torch, lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True, mfma16=True), 3)
    clocks["mfma16_register_loop_random_operands"] = clock_during(
        lambda: B.k_mfma_probe(512, 10000, sink, random_operands=True, mfma16=True), 4, int(3e6 * sec_probe_16))
    clocks["whole_step"] = clock_during(step, 3, int(2e6 * sec_step))
    src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    sec_copy, _ = timed(torch, lambda: B.k_copy(src, dst), 3)
    del src, dst, sink
    return {"variant_cached_teacher_logits": variant, "teacher_microbatch_sweep": sweep, "student_adamw_step": adamw,
            "measured_references": {"mfma_register_loop_tflops": probe_flops / sec_probe / 1e12,
                                    "mfma_register_loop_random_operands_tflops": probe_flops / sec_probe_r / 1e12,
                                    "mfma16_register_loop_random_operands_tflops": probe_flops / sec_probe_16 / 1e12,
                                    "shader_clock_mhz": clocks,
                                    "copy_1gib_read_plus_write_gbs": 2.0 * (1 << 30) / sec_copy / 1e9}}


def bench_secondary(name, args, torch, B, wl, dev):
    """c3: the KD head alone on given hidden states; c4: one vision-encoder section forward+backward on a packed
    micro-batch of image samples.  Same timing protocol as the KD step."""
    work = wl.workload(name, 0)
    dt = torch.bfloat16
    att = (0.0, 0.0)
    if work.student is None:
        kd, n = work.kd, work.n_tokens
        h_t = wl.normal(0, "c3.ht", (n, kd.h_teacher), 1.0, 0.0, dt, dev)
        h_s = wl.normal(0, "c3.hs", (n, kd.h_student), 1.0, 0.0, dt, dev)
        wt = wl.normal(0, "c3.wt", (kd.vocab, kd.h_teacher), 0.02, 0.0, dt, dev)
        ws = wl.normal(0, "c3.ws", (kd.vocab, kd.h_student), 0.02, 0.0, dt, dev)
        d_ws = torch.zeros((kd.vocab, kd.h_student), dtype=torch.float32, device=dev)
        wsb = B.workspace(B.kd_workspace_bytes(kd, n), dev, "kd")
        fn = lambda: B.kd_loss_forward_backward(kd, wt, ws, h_t, h_s, d_w_student=d_ws, ws=wsb)
        flops = kd_flops(kd, n)
        what = "KD head (both lm_heads, KL loss, gradients to student hidden states and lm_head)"
        desc = f"{work.name}: {what}, {n} tokens, vocab {kd.vocab} in chunks of {kd.chunk}, hidden {kd.h_teacher}/{kd.h_student}, T={kd.temperature:g}"
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
        flops = section_flops(cfg, n, pairs, True)
        a = 4.0 * cfg.n_q_heads * cfg.head_dim * pairs * cfg.n_layers
        att = (a, 2.5 * a)
        desc = (f"{work.name}: vision-encoder section forward+backward, {n} packed patch tokens, {batch.n_seqs} image samples "
                f"(max {batch.max_seqlen}), {describe(cfg)}, bidirectional")
    progress(args, f"{name}: inputs and weights resident, first launch next")
    for _ in range(args.warmup):
        fn()
    torch.cuda.synchronize()
    progress(args, f"{name}: warm-up done")
    sec, _ = timed(torch, fn, args.steps)
    progress(args, f"{name}: timed steps done")
    if args.dispatch_only:
        return {"workload": work.name, "n_tokens": n, "ms_per_step": 1e3 * sec}
    prof_steps = min(args.steps, 2)
    prof = profile_steps(torch, B, fn, prof_steps)
    return {"workload": desc, "n_tokens": n, "ms_per_step": 1e3 * sec, "tokens_per_s": n / sec,
            "model_tflop_per_step": flops / 1e12, "mfma_frac_whole_step": flops / sec / 1e12 / PEAK_BF16_TFLOPS,
            "kernels": kernel_table(prof, prof_steps, att)}


def cpu_baseline(work, tw, sw, wt, ws, ids, sample_tokens):
    """The oracle as it stands, timed on the first `sample_tokens` tokens of the same batch
    (sequences truncated to fit), all host threads numpy's BLAS uses."""
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
            "sample": f"first {tot} tokens of the {work.name} batch ({len(lens)} sequence(s)), full model widths and vocab, "
                      f"{sec:.1f} s of fp64 numpy work", "loss": out["loss"]}


def wavefront_schedule(B, wl, vit, llm):
    """Sec. 3.4 closed on measured rates: the 64 samples of the c4 mix go through a vision-encoder section (c4's
    layers) in front of a critical LLM section (c5's student layers); each sample's six times are its model flops
    in each section divided by the rate this library just measured for that section (forward : backward flops =
    1 : 2 for the linears, 1 : 2.5 for attention).  A sample's LLM tokens = its visual tokens after the 4:1 merge plus
    a seeded text length in [256, 2048] (the workload names no text lengths: a reading); text-only samples skip the
    vision section (zero times there).  Reports the simulated makespan in input order and in the scheduler's order."""
    work = wl.workload("c4", 0)
    v_cfg, l_cfg = work.student, wl.workload("c5", 0).student
    text = [int(t) for t in wl.randint(0, "c4.text_lengths", len(work.lengths), 256, 2049).tolist()]
    v_rate = vit["model_tflop_per_step"] / vit["ms_per_step"] * 1e15      # flop/s of the encoder section, fwd+bwd
    l_rate = llm["student_section_tflops"] * 1e12

    def fb(cfg, tokens, pairs):
        g = 2.0 * cfg.layer_params() * tokens * cfg.n_layers
        a = 4.0 * cfg.n_q_heads * cfg.head_dim * pairs * cfg.n_layers
        return g + a, 2.0 * g + 2.5 * a
    tuples = []
    for lv, lt in zip(work.lengths, text):
        vf, vb = fb(v_cfg, lv, lv * lv)
        n_llm = lv // 4 + lt
        lf, lb = fb(l_cfg, n_llm, n_llm * (n_llm + 1) // 2)
        tuples.append((vf / v_rate, lf / l_rate, 0.0, 0.0, lb / l_rate, vb / v_rate))
    order, mk = B.schedule_samples(tuples, interleave=True)
    mk_in, idle_in = B.schedule_makespan(tuples, list(range(len(tuples))), interleave=True)
    mk_s, idle_s = B.schedule_makespan(tuples, order, interleave=True)
    crit = sum(t[1] + t[4] for t in tuples)
    return {"samples": len(tuples), "text_only": sum(1 for l in work.lengths if l == 0),
            "rates_tflops": {"vision_section_fwd_bwd": v_rate / 1e12, "llm_section_fwd_bwd": l_rate / 1e12},
            "critical_section_busy_ms": 1e3 * crit,
            "input_order": {"makespan_ms": 1e3 * mk_in, "critical_idle_ms": 1e3 * idle_in},
            "scheduled_order": {"makespan_ms": 1e3 * mk_s, "critical_idle_ms": 1e3 * idle_s, "first_samples": order[:8]},
            "makespan_ratio": mk_s / mk_in}


def as_line(res, args, metric):
    line = {"metric": metric, "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": {"workload": res["workload"]}}
    line.update({k: v for k, v in res.items() if k not in ("workload", "tokens_per_s", "ms_per_step")})
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all", choices=["all", "c2", "c3", "c4", "c5"],
                    help="all: headline c5 with c2, c3, c4 as sub-objects; else that workload alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0: 1024 for c5, 2048 for c2")
    ap.add_argument("--step-only", action="store_true",
                    help="skip the side measurements (KD head alone, teacher sweep, AdamW, references): for profiler runs of the step")
    ap.add_argument("--dispatch-only", action="store_true",
                    help="run the warm-up and the timed steps of one workload and print a short line: no per-kernel "
                         "events, no side measurements (for profiler counter runs, which only need the dispatches)")
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
    progress(args, "library loaded, GPU visible")
    dev = "cuda"
    kd_metric = "KD step tokens/s (teacher fwd + student fwd+bwd + fused KL loss), 1 GPU"

    def free():
        B._ws_cache.clear()
        torch.cuda.empty_cache()

    def run_one(name, head):
        args.cpu_baseline_here = head and not args.no_cpu_baseline and name in ("c2", "c5")
        if not args.cpu_sample_tokens:
            args.cpu_sample_tokens = 1024 if name == "c5" else 2048
        if name in ("c2", "c5"):
            return bench_kd_step(name, args, torch, B, wl, dev, side=(name == "c2"))
        return bench_secondary(name, args, torch, B, wl, dev)

    if args.dispatch_only:
        if args.workload == "all":
            print("--dispatch-only needs one --workload", file=sys.stderr)
            sys.exit(2)
        args.no_cpu_baseline = True
        print(json.dumps(run_one(args.workload, True)))
        return
    if args.workload != "all":
        res = run_one(args.workload, True)
        metric = kd_metric if args.workload in ("c2", "c5") else res["workload"].split(":")[1].split(",")[0].strip() + " tokens/s, 1 GPU"
        print(json.dumps(as_line(res, args, metric)))
        return
    head = run_one("c5", True)
    free()
    others = {}
    for name in ("c2", "c3", "c4"):
        others[name] = run_one(name, False)
        free()
    line = as_line(head, args, kd_metric)
    line["workloads"] = others
    line["wavefront_schedule_c4_mix"] = wavefront_schedule(B, wl, others["c4"], head)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
