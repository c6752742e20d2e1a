"""Section forward / backward over a packed micro-batch (oracle).

A section is a stack of identical transformer layers with an execution mode:
the teacher section runs forward only, the student (or vision-encoder) section
runs forward and backward (paper Sec. 2.2; Sec. 3.1 for what a section groups).
Pre-norm layers:

  decoder:  x2 = x + Wo attn(rope(Wqkv rmsnorm(x)));  y = x2 + Wd swiglu(Wgu rmsnorm(x2))
  encoder:  same skeleton with LayerNorm, biases, exact GELU, no RoPE, no mask

and a final norm produces the hidden states that leave the section (only
hidden states, never logits, cross a section boundary: Sec. 3.1).

`rnd` is applied exactly where the bf16 HIP path stores a tensor between
kernels; `rnd_res` (default: the same as `rnd`) is applied to the residual
stream (layer inputs / outputs and the post-attention sum), which a path may
keep in higher precision than the other activations.  In the backward pass
`rnd` is also the rounding of the attention probabilities and score gradients
where they enter a matrix product as operands (attention_bwd's `rnd_p`).  With
`rnd=identity` everything is plain float64.
"""
from dataclasses import dataclass

import numpy as np

from . import ops
from .attention import attention_bwd, attention_fwd
from .rounding import identity


@dataclass
class SectionSpec:
    arch: str            # "decoder" or "encoder"
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int = 0       # 0: the section is fed embeddings [N, d_model], else token ids
    norm_eps: float = 1e-6
    rope_base: float = 1e4


def _norm_fwd(spec, x, g, b):
    if spec.arch == "decoder":
        y, r = ops.rmsnorm_fwd(x, g, spec.norm_eps)
        return y, (None, r)
    y, mu, r = ops.layernorm_fwd(x, g, b, spec.norm_eps)
    return y, (mu, r)


def _norm_bwd(spec, dy, x, stats, g):
    mu, r = stats
    if spec.arch == "decoder":
        dx, dg = ops.rmsnorm_bwd(dy, x, r, g)
        return dx, dg, None
    return ops.layernorm_bwd(dy, x, mu, r, g)


def section_forward(spec, weights, cu_seqlens, x_in, rnd=identity, keep=False, rnd_res=None):
    """Returns h_out[N, d] (and the per-layer activations if keep=True)."""
    rnd_res = rnd if rnd_res is None else rnd_res
    dec = spec.arch == "decoder"
    nq, nkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    if spec.vocab > 0:
        x = rnd_res(ops.embedding_fwd(x_in, weights["embedding"]))
    else:
        x = np.asarray(x_in, dtype=np.float64)
    n = x.shape[0]
    pos = ops.positions_from_cu(cu_seqlens)
    stash = []
    for lw in weights["layers"]:
        h1, st1 = _norm_fwd(spec, x, lw["norm1_g"], lw.get("norm1_b"))
        h1 = rnd(h1)
        qkv = rnd(ops.linear_fwd(h1, lw["w_qkv"], lw.get("b_qkv")))
        q = qkv[:, :nq * hd].reshape(n, nq, hd)
        k = qkv[:, nq * hd:(nq + nkv) * hd].reshape(n, nkv, hd)
        v = qkv[:, (nq + nkv) * hd:].reshape(n, nkv, hd)
        if dec:
            q = rnd(ops.rope_apply(q, pos, spec.rope_base))
            k = rnd(ops.rope_apply(k, pos, spec.rope_base))
        o = rnd(attention_fwd(q, k, v, cu_seqlens, causal=dec)).reshape(n, nq * hd)
        x2 = rnd_res(x + ops.linear_fwd(o, lw["w_o"], lw.get("b_o")))
        h2, st2 = _norm_fwd(spec, x2, lw["norm2_g"], lw.get("norm2_b"))
        h2 = rnd(h2)
        up = rnd(ops.linear_fwd(h2, lw["w_up"], lw.get("b_up")))
        a = rnd(ops.swiglu_fwd(up) if dec else ops.gelu_fwd(up))
        y = rnd_res(x2 + ops.linear_fwd(a, lw["w_down"], lw.get("b_down")))
        if keep:
            stash.append(dict(x=x, st1=st1, h1=h1, q=q, k=k, v=v, o=o, x2=x2, st2=st2, h2=h2, up=up, a=a))
        x = y
    h_out, stf = _norm_fwd(spec, x, weights["final_norm_g"], weights.get("final_norm_b"))
    h_out = rnd(h_out)
    if keep:
        return h_out, dict(layers=stash, y_last=x, stf=stf, pos=pos, x_in=x_in)
    return h_out


def section_backward(spec, weights, cu_seqlens, cache, d_h_out, rnd=identity, rnd_res=None):
    """Given dL/dh_out returns (grads, d_x_in): grads mirrors `weights` (float64,
    not rounded: weight gradients are accumulated in high precision), d_x_in is
    the gradient w.r.t. the input embeddings (None for a token-id section, whose
    input gradient is the embedding-table gradient)."""
    rnd_res = rnd if rnd_res is None else rnd_res
    dec = spec.arch == "decoder"
    nq, nkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    n = d_h_out.shape[0]
    grads = {"layers": [None] * spec.n_layers}
    dy, dg, db = _norm_bwd(spec, d_h_out, cache["y_last"], cache["stf"], weights["final_norm_g"])
    grads["final_norm_g"], grads["final_norm_b"] = dg, db
    dy = rnd_res(dy)
    for li in range(spec.n_layers - 1, -1, -1):
        lw, c = weights["layers"][li], cache["layers"][li]
        g = {}
        bias = not dec
        da, g["w_down"], g["b_down"] = ops.linear_bwd(dy, c["a"], lw["w_down"], bias)
        da = rnd(da)
        dup = rnd(ops.swiglu_bwd(da, c["up"]) if dec else ops.gelu_bwd(da, c["up"]))
        dh2, g["w_up"], g["b_up"] = ops.linear_bwd(dup, c["h2"], lw["w_up"], bias)
        dh2 = rnd(dh2)
        dn, g["norm2_g"], g["norm2_b"] = _norm_bwd(spec, dh2, c["x2"], c["st2"], lw["norm2_g"])
        dx2 = rnd_res(dy + dn)
        do, g["w_o"], g["b_o"] = ops.linear_bwd(dx2, c["o"], lw["w_o"], bias)
        do = rnd(do).reshape(n, nq, hd)
        dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], cu_seqlens, causal=dec,
                                   o=c["o"].reshape(n, nq, hd), rnd_p=rnd)
        dq, dk, dv = rnd(dq), rnd(dk), rnd(dv)
        if dec:
            dq = rnd(ops.rope_apply(dq, cache["pos"], spec.rope_base, inverse=True))
            dk = rnd(ops.rope_apply(dk, cache["pos"], spec.rope_base, inverse=True))
        dqkv = np.concatenate([dq.reshape(n, -1), dk.reshape(n, -1), dv.reshape(n, -1)], axis=1)
        dh1, g["w_qkv"], g["b_qkv"] = ops.linear_bwd(dqkv, c["h1"], lw["w_qkv"], bias)
        dh1 = rnd(dh1)
        dn, g["norm1_g"], g["norm1_b"] = _norm_bwd(spec, dh1, c["x"], c["st1"], lw["norm1_g"])
        dy = rnd_res(dx2 + dn)
        grads["layers"][li] = g
    if spec.vocab > 0:
        grads["embedding"] = ops.embedding_bwd(cache["x_in"], dy, spec.vocab)
        return grads, None
    return grads, dy
