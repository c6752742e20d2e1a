"""Layer-level building blocks of the oracle, forward and explicit backward.

The paper inherits its per-GPU transformer compute from an existing training
framework and states no layer equations (Sec. 4, experimental setup); the
definitions here are the textbook ones fixed by the workload configs:
RMSNorm / RoPE / SwiGLU for decoder sections, LayerNorm / GELU for encoder
sections, weights stored `[out, in]`.  All arithmetic is float64.
"""
import numpy as np
from scipy.special import erf


# ----------------------------------------------------------------- linear
def linear_fwd(x, w, b=None):
    """y[t, o] = sum_i x[t, i] w[o, i] (+ b[o])."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def linear_bwd(dy, x, w, has_bias=False):
    """dx = dy W,  dW = dy^T x,  db = sum_t dy."""
    dx = dy @ w
    dw = dy.T @ x
    db = dy.sum(axis=0) if has_bias else None
    return dx, dw, db


# ----------------------------------------------------------------- norms
def rmsnorm_fwd(x, g, eps):
    """y = x * r * g with r = (mean_j x_j^2 + eps)^(-1/2); returns (y, r)."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=1) + eps)
    return x * r[:, None] * g[None, :], r


def rmsnorm_bwd(dy, x, r, g):
    """dg = sum_t dy*xhat;  dx = r (dy*g - xhat mean_j(dy*g*xhat))."""
    xh = x * r[:, None]
    dg = np.sum(dy * xh, axis=0)
    t = dy * g[None, :]
    dx = r[:, None] * (t - xh * np.mean(t * xh, axis=1)[:, None])
    return dx, dg


def layernorm_fwd(x, g, b, eps):
    """y = (x - mu) * r * g + b, r = (biased var + eps)^(-1/2); returns (y, mu, r)."""
    mu = np.mean(x, axis=1)
    xc = x - mu[:, None]
    r = 1.0 / np.sqrt(np.mean(xc * xc, axis=1) + eps)
    return xc * r[:, None] * g[None, :] + b[None, :], mu, r


def layernorm_bwd(dy, x, mu, r, g):
    """dx = r (t - mean(t) - xhat mean(t*xhat)), t = dy*g; dg = sum dy*xhat; db = sum dy."""
    xh = (x - mu[:, None]) * r[:, None]
    dg = np.sum(dy * xh, axis=0)
    db = np.sum(dy, axis=0)
    t = dy * g[None, :]
    dx = r[:, None] * (t - np.mean(t, axis=1)[:, None] - xh * np.mean(t * xh, axis=1)[:, None])
    return dx, dg, db


# ----------------------------------------------------------------- RoPE
def positions_from_cu(cu_seqlens):
    """Position of every packed token inside its own sequence (restarts at 0)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    n = int(cu[-1])
    pos = np.zeros(n, dtype=np.int64)
    for b in range(len(cu) - 1):
        pos[cu[b]:cu[b + 1]] = np.arange(cu[b + 1] - cu[b])
    return pos


def rope_apply(x, pos, base, inverse=False):
    """Half-split rotary embedding on x[N, heads, hd].

    Pair (i, i + hd/2) of every head is rotated by the angle pos * base^(-2i/hd);
    `inverse=True` rotates by the negative angle, which is the backward pass
    (the transpose of a rotation).
    """
    hd = x.shape[-1]
    half = hd // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = pos.astype(np.float64)[:, None] * theta[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    if inverse:
        s = -s
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# ----------------------------------------------------------------- activations
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def swiglu_fwd(gu):
    """gu = [gate | up] along features; a = gate * sigmoid(gate) * up."""
    f = gu.shape[1] // 2
    g, u = gu[:, :f], gu[:, f:]
    return g * sigmoid(g) * u


def swiglu_bwd(da, gu):
    f = gu.shape[1] // 2
    g, u = gu[:, :f], gu[:, f:]
    s = sigmoid(g)
    dg = da * u * s * (1.0 + g * (1.0 - s))
    du = da * g * s
    return np.concatenate([dg, du], axis=1)


def gelu_fwd(x):
    """Exact (erf) GELU: x * Phi(x)."""
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_bwd(dy, x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    cdf = 0.5 * (1.0 + erf(x / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return dy * (cdf + x * pdf)


# ----------------------------------------------------------------- embedding
def embedding_fwd(ids, table):
    return table[np.asarray(ids, dtype=np.int64)]


def embedding_bwd(ids, dx, vocab):
    """dE[id[t], :] += dx[t, :] (repeated ids accumulate)."""
    de = np.zeros((vocab, dx.shape[1]), dtype=np.float64)
    np.add.at(de, np.asarray(ids, dtype=np.int64), dx)
    return de
