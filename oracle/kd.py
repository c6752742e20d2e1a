"""Temperature-softmax KL distillation loss on logits (oracle).

The student section holds the teacher's output layer as well as its own, so
the loss consumes two hidden-state tensors and two lm_head matrices and the
logits exist only inside it (paper Sec. 3.1, section construction for KL-based
distillation; Sec. 4.2).  The teacher is frozen: no gradient reaches it
(Sec. 2.2).

  z_t = h_t Wt^T,  z_s = h_s Ws^T,  p = softmax(z_t / T),  q = softmax(z_s / T)
  KL_tok = sum_v p_v (ln p_v - ln q_v),      loss = loss_scale * sum_tok KL_tok
  dz_s = (loss_scale / T) (q - p),  dh_s = dz_s Ws,  dWs = dz_s^T h_s

Full `[block, V]` logits are formed for blocks of tokens (tokens are
independent, so blocking over tokens changes nothing); there is no blocking
over the vocabulary.
"""
import numpy as np

from .rounding import identity


def _log_softmax(z):
    m = np.max(z, axis=1, keepdims=True)
    return z - m - np.log(np.sum(np.exp(z - m), axis=1, keepdims=True))


def kd_loss_forward_backward(h_t, h_s, w_t, w_s, temperature, loss_scale,
                             rnd=identity, need_grad=True, token_block=1024):
    """Returns dict(loss, kl_tok[N], d_h_s[N, Hs], d_w_s[V, Hs]).

    `rnd` rounds the logit gradient dz_s (the tensor the bf16 path stores
    between the softmax-difference step and the two gradient GEMMs) and d_h_s.
    """
    n = h_s.shape[0]
    kl_tok = np.zeros(n, dtype=np.float64)
    d_h_s = np.zeros_like(h_s) if need_grad else None
    d_w_s = np.zeros_like(w_s) if need_grad else None
    for t0 in range(0, n, token_block):
        t1 = min(n, t0 + token_block)
        lp = _log_softmax((h_t[t0:t1] @ w_t.T) / temperature)
        lq = _log_softmax((h_s[t0:t1] @ w_s.T) / temperature)
        p = np.exp(lp)
        kl_tok[t0:t1] = np.sum(p * (lp - lq), axis=1)
        if need_grad:
            dz = rnd((loss_scale / temperature) * (np.exp(lq) - p))
            d_h_s[t0:t1] = dz @ w_s
            d_w_s += dz.T @ h_s[t0:t1]
    out = dict(loss=loss_scale * float(np.sum(kl_tok)), kl_tok=kl_tok)
    if need_grad:
        out["d_h_s"] = rnd(d_h_s)
        out["d_w_s"] = d_w_s
    return out
