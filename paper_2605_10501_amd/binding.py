"""Thin ctypes binding of libmaestro_section.so (same names as the C ABI, minus the ms_ prefix).

Argument marshalling only: every step of the path runs inside the HIP library.  PyTorch
provides device memory and the current stream.  There is no CPU fallback: if the library is
missing, loading fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmaestro_section.so")
MS_F32, MS_BF16 = 0, 1
MS_DECODER, MS_ENCODER = 0, 1
_LAYER_FIELDS = ["norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "norm2_g", "norm2_b", "w_up", "b_up", "w_down", "b_down"]


class SectionConfigC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ["arch", "dtype", "n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab"]] + [("norm_eps", C.c_float), ("rope_base", C.c_float)]


class LayerPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class SectionPtrs(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("layers", C.POINTER(LayerPtrs)),
                ("final_norm_g", C.c_void_p), ("final_norm_b", C.c_void_p)]


class BatchC(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("n_seqs", C.c_int32),
                ("cu_seqlens_dev", C.c_void_p), ("cu_seqlens_host", C.POINTER(C.c_int32))]


class KDConfigC(C.Structure):
    _fields_ = [("vocab", C.c_int32), ("h_teacher", C.c_int32), ("h_student", C.c_int32), ("chunk", C.c_int32),
                ("dtype", C.c_int32), ("temperature", C.c_float), ("loss_scale", C.c_float),
                ("w_teacher_dev", C.c_void_p), ("w_student_dev", C.c_void_p), ("token_block", C.c_int32)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2605_10501_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_10501_amd.build`")
        _lib = C.CDLL(LIB_PATH)
        _lib.ms_last_error.restype = C.c_char_p
        for name in ["ms_section_workspace_bytes", "ms_kd_workspace_bytes", "ms_k_norm_backward_scratch_bytes",
                     "ms_k_attention_backward_scratch_bytes"]:
            getattr(_lib, name).restype = C.c_size_t
    return _lib


def _check(status):
    if status != 0:
        raise RuntimeError(f"maestro_section error {status}: {lib().ms_last_error().decode()}")


def _p(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(dtype):
    if dtype in ("bf16", torch.bfloat16, MS_BF16):
        return MS_BF16
    if dtype in ("fp32", torch.float32, MS_F32) and dtype is not False:
        return MS_F32
    raise ValueError(dtype)


def _tdt(dtype):
    return torch.bfloat16 if _dt(dtype) == MS_BF16 else torch.float32


class Batch:
    """A packed micro-batch: host and device copies of cu_seqlens."""

    def __init__(self, cu_seqlens, device="cuda"):
        self.cu = [int(v) for v in cu_seqlens]
        self.n_seqs = len(self.cu) - 1
        self.n_tokens = self.cu[-1] if self.cu else 0
        self.max_seqlen = max([b - a for a, b in zip(self.cu[:-1], self.cu[1:])], default=0)
        self._host = (C.c_int32 * len(self.cu))(*self.cu)
        self.cu_dev = torch.tensor(self.cu, dtype=torch.int32, device=device)

    def c(self):
        return BatchC(self.n_tokens, self.n_seqs, _p(self.cu_dev), self._host)


def _cfg_c(cfg):
    return SectionConfigC(MS_DECODER if cfg.arch == "decoder" else MS_ENCODER, _dt(cfg.dtype), cfg.n_layers, cfg.d_model,
                          cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.norm_eps, cfg.rope_base)


def _ptrs_c(cfg, w):
    layers = (LayerPtrs * cfg.n_layers)()
    for i, lw in enumerate(w["layers"]):
        for f in _LAYER_FIELDS:
            t = lw.get(f)
            setattr(layers[i], f, t.data_ptr() if t is not None else None)
    emb, fb = w.get("embedding"), w.get("final_norm_b")
    s = SectionPtrs(emb.data_ptr() if emb is not None else None, layers, w["final_norm_g"].data_ptr(),
                    fb.data_ptr() if fb is not None else None)
    s._keep = layers
    return s


def _kd_c(kd, w_teacher, w_student, loss_scale):
    return KDConfigC(kd.vocab, kd.h_teacher, kd.h_student, kd.chunk, _dt(kd.dtype), kd.temperature, loss_scale,
                     w_teacher.data_ptr(), w_student.data_ptr(), getattr(kd, "token_block", 0))


def zero_grads(weights):
    """fp32 zero buffers with the structure of `weights`."""
    def z(t):
        return torch.zeros(t.shape, dtype=torch.float32, device=t.device) if t is not None else None
    g = {k: z(v) for k, v in weights.items() if k != "layers"}
    g["layers"] = [{k: z(v) for k, v in lw.items()} for lw in weights["layers"]]
    return g


_ws_cache = {}


def workspace(nbytes, device="cuda", tag="default"):
    """A cached byte buffer of at least nbytes (grown on demand)."""
    buf = _ws_cache.get(tag)
    if buf is None or buf.numel() < nbytes:
        _ws_cache[tag] = buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    return buf


def section_workspace_bytes(cfg, max_tokens, max_seqlen, need_backward):
    c = _cfg_c(cfg)
    return lib().ms_section_workspace_bytes(C.byref(c), max_tokens, max_seqlen, int(need_backward))


def kd_workspace_bytes(kd, max_tokens):
    c = KDConfigC(kd.vocab, kd.h_teacher, kd.h_student, kd.chunk, _dt(kd.dtype), kd.temperature, 1.0, None, None,
                  getattr(kd, "token_block", 0))
    return lib().ms_kd_workspace_bytes(C.byref(c), max_tokens)


def section_forward(cfg, weights, batch, x_in, h_out=None, ws=None):
    c, w, b = _cfg_c(cfg), _ptrs_c(cfg, weights), batch.c()
    if h_out is None:
        h_out = torch.empty((batch.n_tokens, cfg.d_model), dtype=_tdt(cfg.dtype), device=x_in.device)
    if ws is None:
        ws = workspace(section_workspace_bytes(cfg, batch.n_tokens, batch.max_seqlen, False), x_in.device)
    _check(lib().ms_section_forward(C.byref(c), C.byref(w), C.byref(b), _p(x_in), _p(h_out), _p(ws),
                                    C.c_size_t(ws.numel()), _stream()))
    return h_out


def section_forward_backward(cfg, weights, grads, batch, x_in, d_h_out=None, kd=None, w_teacher=None, w_student=None,
                             h_teacher=None, d_w_student=None, loss_scale=None, want_d_x_in=False, ws=None):
    """Returns dict(h_out, loss, kl_tok, d_x_in); `grads` (and d_w_student) are accumulated in place."""
    c, w, g, b = _cfg_c(cfg), _ptrs_c(cfg, weights), _ptrs_c(cfg, grads), batch.c()
    dev, n = x_in.device, batch.n_tokens
    h_out = torch.empty((n, cfg.d_model), dtype=_tdt(cfg.dtype), device=dev)
    need = section_workspace_bytes(cfg, n, batch.max_seqlen, True)
    loss = kl = kdc = None
    if kd is not None:
        kdc = _kd_c(kd, w_teacher, w_student, (1.0 / max(n, 1)) if loss_scale is None else loss_scale)
        need += kd_workspace_bytes(kd, n)
        loss = torch.zeros((), dtype=torch.float32, device=dev)
        kl = torch.empty((n,), dtype=torch.float32, device=dev)
    d_x_in = torch.empty_like(h_out) if (want_d_x_in and cfg.vocab == 0) else None
    if ws is None:
        ws = workspace(need, dev)
    _check(lib().ms_section_forward_backward(
        C.byref(c), C.byref(w), C.byref(g), C.byref(b), _p(x_in), _p(h_out), _p(d_h_out),
        C.byref(kdc) if kdc is not None else None, _p(h_teacher), _p(d_w_student), _p(loss), _p(kl), _p(d_x_in),
        _p(ws), C.c_size_t(ws.numel()), _stream()))
    return dict(h_out=h_out, loss=loss, kl_tok=kl, d_x_in=d_x_in)


def kd_loss_forward_backward(kd, w_teacher, w_student, h_teacher, h_student, loss_scale=None, need_d_h=True,
                             d_w_student=None, ws=None):
    """Returns dict(loss, kl_tok, d_h_s); d_w_student (fp32 [V, Hs]) is accumulated in place if given."""
    n, dev = h_student.shape[0], h_student.device
    kdc = _kd_c(kd, w_teacher, w_student, (1.0 / max(n, 1)) if loss_scale is None else loss_scale)
    loss = torch.zeros((), dtype=torch.float32, device=dev)
    kl = torch.empty((n,), dtype=torch.float32, device=dev)
    d_h = torch.empty_like(h_student) if need_d_h else None
    if ws is None:
        ws = workspace(kd_workspace_bytes(kd, n), dev)
    _check(lib().ms_kd_loss_forward_backward(C.byref(kdc), n, _p(h_teacher), _p(h_student), _p(loss), _p(kl), _p(d_h),
                                             _p(d_w_student), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return dict(loss=loss, kl_tok=kl, d_h_s=d_h)


KD_STATIC_SCRATCH_BYTES = 64 << 20


def kd_loss_forward_backward_static(kd, w_teacher, w_student, h_teacher, h_student, loss, kl_tok, d_h_student,
                                    d_w_student=None, loss_scale=None):
    """The allocation-free variant: every output is the caller's tensor, the scratch is the library's built-in array."""
    n = h_student.shape[0]
    kdc = _kd_c(kd, w_teacher, w_student, (1.0 / max(n, 1)) if loss_scale is None else loss_scale)
    _check(lib().ms_kd_loss_forward_backward_static(C.byref(kdc), n, _p(h_teacher), _p(h_student), _p(loss), _p(kl_tok),
                                                    _p(d_h_student), _p(d_w_student), _stream()))


def pack_microbatches(lengths, token_budget, policy=0):
    """Returns (order, mb_offsets, cu_seqlens_per_mb) as Python lists."""
    n = len(lengths)
    arr = (C.c_int32 * max(n, 1))(*lengths)
    order, offs, cus = (C.c_int32 * max(n, 1))(), (C.c_int32 * (n + 1))(), (C.c_int32 * max(2 * n, 1))()
    n_mb = C.c_int32(0)
    _check(lib().ms_pack_microbatches(arr, n, token_budget, policy, order, offs, C.byref(n_mb), cus))
    offs_l = [offs[i] for i in range(n_mb.value + 1)]
    out, pos = [], 0
    for m in range(n_mb.value):
        k = offs_l[m + 1] - offs_l[m]
        out.append([cus[pos + i] for i in range(k + 1)])
        pos += k + 1
    return [order[i] for i in range(offs_l[-1])], offs_l, out


class _MergerCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("d_vit", C.c_int32), ("merge", C.c_int32), ("d_hidden", C.c_int32), ("d_llm", C.c_int32)]


class _MergerPtrs(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("w1", "b1", "w2", "b2")]


def _merger_c(w, merge):
    dh, din = w["w1"].shape
    return _MergerCfg(_dt(w["w1"].dtype), din // merge, merge, dh, w["w2"].shape[0])


def _merger_ptrs(t):
    return _MergerPtrs(*[_p(t[k]) for k in ("w1", "b1", "w2", "b2")])


def merger_workspace_bytes(w, n_groups, merge=4):
    c = _merger_c(w, merge)
    lib().ms_merger_workspace_bytes.restype = C.c_size_t
    return lib().ms_merger_workspace_bytes(C.byref(c), n_groups)


def merger_forward(w, h_vit, positions, x_llm, ws, merge=4):
    """Writes the projected visual rows into x_llm (in place) at `positions` (int32 device tensor)."""
    c, pw = _merger_c(w, merge), _merger_ptrs(w)
    _check(lib().ms_merger_forward(C.byref(c), C.byref(pw), positions.numel(), _p(h_vit), _p(positions), x_llm.shape[0], _p(x_llm),
                                   _p(ws), C.c_size_t(ws.numel()), _stream()))


def merger_backward(w, grads, h_vit, positions, d_x_llm, ws, merge=4):
    """Returns d_h_vit; `grads` (fp32 dict like w) is accumulated in place.  `ws` must be the forward call's workspace."""
    c, pw, pg = _merger_c(w, merge), _merger_ptrs(w), _merger_ptrs(grads)
    d_h = torch.empty_like(h_vit)
    _check(lib().ms_merger_backward(C.byref(c), C.byref(pw), C.byref(pg), positions.numel(), _p(h_vit), _p(positions),
                                    d_x_llm.shape[0], _p(d_x_llm), _p(d_h), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return d_h


class _AdamWCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("grad_scale", C.c_float), ("step", C.c_int32), ("zero_grad", C.c_int32)]


def adamw_step(grad, master, m, v, weight, step, lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, grad_scale=1.0,
               zero_grad=False):
    """In-place AdamW update of fp32 master / m / v from fp32 grad; `weight` (bf16 or fp32, or None) gets round(master)."""
    cfg = _AdamWCfg(lr, beta1, beta2, eps, weight_decay, grad_scale, step, int(zero_grad))
    dt = MS_F32 if weight is None else _dt(weight.dtype)
    _check(lib().ms_adamw_step(C.byref(cfg), dt, C.c_int64(master.numel()), _p(grad), _p(master), _p(m), _p(v), _p(weight),
                               _stream()))


def schedule_samples(tuples, interleave=True):
    """tuples: n x 6 times (Sec. 3.4).  Returns (order, makespan)."""
    n = len(tuples)
    flat = (C.c_double * max(6 * n, 1))(*[float(x) for t in tuples for x in t])
    order, mk = (C.c_int32 * max(n, 1))(), C.c_double(0.0)
    _check(lib().ms_schedule_samples(n, flat, int(bool(interleave)), order, C.byref(mk)))
    return [order[i] for i in range(n)], mk.value


def schedule_makespan(tuples, order, interleave=True):
    """Returns (makespan, critical_idle) of executing `tuples` in `order`."""
    n = len(tuples)
    flat = (C.c_double * max(6 * n, 1))(*[float(x) for t in tuples for x in t])
    arr = (C.c_int32 * max(n, 1))(*order)
    mk, idle = C.c_double(0.0), C.c_double(0.0)
    _check(lib().ms_schedule_makespan(n, flat, arr, int(bool(interleave)), C.byref(mk), C.byref(idle)))
    return mk.value, idle.value


# ------------------------------------------------------------------ kernel-level entry points
def k_gemm_config(tile=0, mfma16=-1):
    """Kernel selection of the bf16 GEMMs (tests, measurements): tile 0 / 128 / 256 / -1, mfma16 -1 / 0 / 1."""
    _check(lib().ms_k_gemm_config(int(tile), int(mfma16)))


def k_gemm(a, b, trans_a=False, trans_b=False, c=None, c_fp32=False, accumulate=False, bias=None, residual=None,
           alpha=1.0, split_k=1, dtype=None):
    res_fp32 = residual is not None and residual.dtype == torch.float32 and a.dtype == torch.bfloat16
    """C[M,N] = alpha * A(m,k) B(n,k) (+bias) (+residual); a / b are 2-D tensors in their stored layout."""
    dt = _dt(dtype if dtype is not None else a.dtype)
    M, K = (a.shape[1], a.shape[0]) if trans_a else a.shape
    N = b.shape[1] if trans_b else b.shape[0]
    if c is None:
        c = torch.empty((M, N), dtype=torch.float32 if (c_fp32 or dt == MS_F32) else torch.bfloat16, device=a.device)
    _check(lib().ms_k_gemm(dt, int(trans_a), int(trans_b), M, N, K, C.c_float(alpha), _p(a), C.c_int64(a.stride(0)),
                           _p(b), C.c_int64(b.stride(0)), _p(c), C.c_int64(c.stride(0)), int(c_fp32), int(accumulate),
                           _p(bias), _p(residual), C.c_int64(residual.stride(0) if residual is not None else 0),
                           int(res_fp32), split_k, _stream()))
    return c


def k_gemm_swiglu(a, w, want_gate_up=True):
    """a[M,K], w[2F,K] (gate rows | up rows) -> (act[M,F], gate_up[M,2F] or None); bf16."""
    M, K = a.shape
    F = w.shape[0] // 2
    act = torch.empty((M, F), dtype=a.dtype, device=a.device)
    gu = torch.empty((M, 2 * F), dtype=a.dtype, device=a.device) if want_gate_up else None
    _check(lib().ms_k_gemm_swiglu(M, F, K, _p(a), C.c_int64(a.stride(0)), _p(w), C.c_int64(w.stride(0)), _p(act),
                                  C.c_int64(F), _p(gu), C.c_int64(2 * F), _stream()))
    return act, gu


def k_norm_forward(kind, x, g, b, eps):
    """x may be fp32 while g / b / y are bf16 (fp32 residual stream of a bf16 section)."""
    n, d = x.shape
    y = torch.empty((n, d), dtype=g.dtype, device=x.device)
    xf = int(x.dtype == torch.float32 and g.dtype == torch.bfloat16)
    rstd = torch.empty(n, dtype=torch.float32, device=x.device)
    mean = torch.empty(n, dtype=torch.float32, device=x.device) if kind == 1 else None
    _check(lib().ms_k_norm_forward(kind, _dt(g.dtype), xf, n, d, C.c_float(eps), _p(x), _p(g), _p(b), _p(y), _p(mean),
                                   _p(rstd), _stream()))
    return y, mean, rstd


def k_norm_backward(kind, dy, x, g, mean, rstd, add=None, dg=None, db=None):
    n, d = x.shape
    dx = torch.empty_like(dy)
    xf = int(x.dtype == torch.float32 and g.dtype == torch.bfloat16)
    dg = torch.zeros(d, dtype=torch.float32, device=x.device) if dg is None else dg
    db = (torch.zeros(d, dtype=torch.float32, device=x.device) if db is None else db) if kind == 1 else None
    sc = workspace(lib().ms_k_norm_backward_scratch_bytes(d), x.device, "norm")
    _check(lib().ms_k_norm_backward(kind, _dt(g.dtype), xf, n, d, _p(dy), _p(x), _p(g), _p(mean), _p(rstd), _p(add), _p(dx),
                                    _p(dg), _p(db), _p(sc), _stream()))
    return dx, dg, db


def k_positions(batch):
    pos = torch.empty(batch.n_tokens, dtype=torch.int32, device=batch.cu_dev.device)
    _check(lib().ms_k_positions(batch.n_tokens, batch.n_seqs, _p(batch.cu_dev), _p(pos), _stream()))
    return pos


def k_rope_table(max_pos, head_dim, base, device="cuda"):
    t = torch.empty((max_pos, head_dim // 2, 2), dtype=torch.float32, device=device)
    _check(lib().ms_k_rope_table(max_pos, head_dim, C.c_float(base), _p(t), _stream()))
    return t


def k_rope(x, n_heads, head_dim, pos, table, inverse=False):
    """In place on x[n, row_stride]."""
    _check(lib().ms_k_rope(_dt(x.dtype), x.shape[0], n_heads, head_dim, C.c_int64(x.stride(0)), _p(x), _p(pos), _p(table),
                           int(inverse), _stream()))
    return x


def k_act_forward(kind, up):
    n, f = up.shape[0], up.shape[1] // 2 if kind == 0 else up.shape[1]
    a = torch.empty((n, f), dtype=up.dtype, device=up.device)
    _check(lib().ms_k_act_forward(kind, _dt(up.dtype), n, f, _p(up), _p(a), _stream()))
    return a


def k_act_backward(kind, da, up):
    dup = torch.empty_like(up)
    _check(lib().ms_k_act_backward(kind, _dt(up.dtype), da.shape[0], da.shape[1], _p(da), _p(up), _p(dup), _stream()))
    return dup


def k_embedding_forward(ids, table, out_fp32=False):
    x = torch.empty((ids.shape[0], table.shape[1]), dtype=torch.float32 if out_fp32 else table.dtype, device=table.device)
    _check(lib().ms_k_embedding_forward(_dt(table.dtype), int(out_fp32), ids.shape[0], table.shape[1], table.shape[0],
                                        _p(ids), _p(table), _p(x), _stream()))
    return x


def k_embedding_backward(ids, dx, vocab, d_table=None):
    if d_table is None:
        d_table = torch.zeros((vocab, dx.shape[1]), dtype=torch.float32, device=dx.device)
    _check(lib().ms_k_embedding_backward(_dt(dx.dtype), ids.shape[0], dx.shape[1], vocab, _p(ids), _p(dx), _p(d_table),
                                         _stream()))
    return d_table


def k_colsum(x, out=None):
    n, c = x.shape
    out = torch.zeros(c, dtype=torch.float32, device=x.device) if out is None else out
    sc = workspace(lib().ms_k_norm_backward_scratch_bytes(c), x.device, "norm")
    _check(lib().ms_k_colsum(_dt(x.dtype), n, c, _p(x), _p(out), _p(sc), _stream()))
    return out


def k_attention_forward(qkv, batch, n_q_heads, n_kv_heads, head_dim, causal):
    n = qkv.shape[0]
    o = torch.empty((n, n_q_heads * head_dim), dtype=qkv.dtype, device=qkv.device)
    lse = torch.empty((n_q_heads, n), dtype=torch.float32, device=qkv.device)
    _check(lib().ms_k_attention_forward(_dt(qkv.dtype), int(causal), n_q_heads, n_kv_heads, head_dim, n, batch.n_seqs,
                                        batch.max_seqlen, _p(batch.cu_dev), _p(qkv), _p(o), _p(lse), _stream()))
    return o, lse


def k_attention_backward(qkv, o, lse, d_o, batch, n_q_heads, n_kv_heads, head_dim, causal):
    n = qkv.shape[0]
    dqkv = torch.empty_like(qkv)
    sc = workspace(lib().ms_k_attention_backward_scratch_bytes(_dt(qkv.dtype), n_q_heads, n_kv_heads, head_dim, n),
                   qkv.device, "attn")
    _check(lib().ms_k_attention_backward(_dt(qkv.dtype), int(causal), n_q_heads, n_kv_heads, head_dim, n, batch.n_seqs,
                                         batch.max_seqlen, _p(batch.cu_dev), _p(qkv), _p(o), _p(lse), _p(d_o), _p(dqkv),
                                         _p(sc), _stream()))
    return dqkv


def k_mfma_probe(workgroups, iters, sink, random_operands=False, mfma16=False):
    _check(lib().ms_k_mfma_probe(workgroups, iters, int(random_operands), int(mfma16), _p(sink), _stream()))


def k_clock_monitor(microseconds, out):
    """out: int64[2] device tensor; launched on the current stream."""
    _check(lib().ms_k_clock_monitor(int(microseconds), _p(out), _stream()))


def k_copy(src, dst):
    _check(lib().ms_k_copy(_p(src), _p(dst), C.c_size_t(src.numel() * src.element_size()), _stream()))
    return dst


PROFILE_CLASSES = ["gemm_nt", "gemm_t", "attn_fwd", "attn_bwd", "norm_fwd", "norm_bwd", "act_fwd", "act_bwd", "rope",
                   "kd_stats", "kd_dz", "misc"]


def profile_enable(on):
    _check(lib().ms_profile_enable(int(on)))


def profile_read():
    """{class name: (launches, total_ms, total_work)} of the launches recorded since profile_enable(1)."""
    out = {}
    for i, name in enumerate(PROFILE_CLASSES):
        n, ms, work = C.c_int64(0), C.c_double(0), C.c_double(0)
        _check(lib().ms_profile_read(i, C.byref(n), C.byref(ms), C.byref(work)))
        out[name] = (n.value, ms.value, work.value)
    return out
