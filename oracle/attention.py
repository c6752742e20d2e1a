"""Dense softmax attention over packed variable-length sequences (oracle).

Each sequence attends only to itself; a decoder section masks keys after the
query (causal), an encoder section does not (the vision encoder of the paper's
Sec. 2.1 attends over the whole visual sequence).  Query head h reads KV head
h // (n_q / n_kv) (grouped-query attention).  The full L x L score matrix is
formed per sequence and head: this is the definition the tiled HIP kernels
re-associate.
"""
import numpy as np

from .rounding import identity


def _softmax_rows(s):
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=1, keepdims=True)


def _scores(qh, kh, causal):
    L, hd = qh.shape
    s = (qh @ kh.T) / np.sqrt(float(hd))
    if causal:
        s = np.where(np.tril(np.ones((L, L), dtype=bool)), s, -np.inf)
    return s


def _probs(qh, kh, causal):
    return _softmax_rows(_scores(qh, kh, causal))


def attention_fwd(q, k, v, cu_seqlens, causal, return_lse=False):
    """q[N, nq, hd], k/v[N, nkv, hd] -> o[N, nq, hd] (and lse[nq, N], the natural-log
    sum of exponentials of each query's visible scaled scores, if return_lse)."""
    n, nq, hd = q.shape
    nkv = k.shape[1]
    grp = nq // nkv
    o = np.zeros_like(q)
    lse = np.zeros((nq, n), dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    for b in range(len(cu) - 1):
        s0, s1 = int(cu[b]), int(cu[b + 1])
        if s1 == s0:
            continue
        for h in range(nq):
            s = _scores(q[s0:s1, h], k[s0:s1, h // grp], causal)
            o[s0:s1, h] = _softmax_rows(s) @ v[s0:s1, h // grp]
            mx = np.max(s, axis=1)
            lse[h, s0:s1] = mx + np.log(np.sum(np.exp(s - mx[:, None]), axis=1))
    return (o, lse) if return_lse else o


def attention_bwd(do, q, k, v, cu_seqlens, causal, o=None, rnd_p=identity):
    """Gradients of attention_fwd: dV = P^T dO, dP = dO V^T,
    dS = P * (dP - delta), dQ = dS K / sqrt(hd), dK = dS^T Q / sqrt(hd);
    dK and dV are summed over the query heads that share a KV head.

    delta is the softmax-Jacobian row term rowsum(dP * P).  Because O = P V it also equals
    rowsum(dO * O); when the stored forward output `o` is passed (the backward pass of a
    section reads the output tensor the forward pass stored, rounded under the bf16
    contract) that second form is used, otherwise the first.

    `rnd_p` is the materialisation rounding of the two score-shaped matrices that enter a
    matrix product as an operand: P in dV = P^T dO, and dS in dQ = dS K and dK = dS^T Q.  A
    path whose matrix units take bf16 operands ("bf16 activations with fp32 accumulation")
    rounds exactly these two; the probabilities inside dS = P * (dP - delta), dP and delta
    stay unrounded.  identity (the default) is the plain definition."""
    n, nq, hd = q.shape
    nkv = k.shape[1]
    grp = nq // nkv
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    scale = 1.0 / np.sqrt(float(hd))
    for b in range(len(cu) - 1):
        s0, s1 = int(cu[b]), int(cu[b + 1])
        if s1 == s0:
            continue
        for h in range(nq):
            g = h // grp
            p = _probs(q[s0:s1, h], k[s0:s1, g], causal)
            doh = do[s0:s1, h]
            dv[s0:s1, g] += rnd_p(p).T @ doh
            dp = doh @ v[s0:s1, g].T
            if o is None:
                delta = np.sum(dp * p, axis=1, keepdims=True)
            else:
                delta = np.sum(doh * o[s0:s1, h], axis=1, keepdims=True)
            ds = rnd_p(p * (dp - delta))
            dq[s0:s1, h] = (ds @ k[s0:s1, g]) * scale
            dk[s0:s1, g] += (ds.T @ q[s0:s1, h]) * scale
    return dq, dk, dv
