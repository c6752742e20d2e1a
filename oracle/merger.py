"""Oracle for the vision -> language hand-off (Sec. 2.1, Sec. 4.1): the encoder's visual tokens are
down-sampled 4:1 along the sequence and joined with the text tokens to form the LLM's input.
TEST INFRASTRUCTURE ONLY: only tests/, the smoke check and the CPU-baseline leg of the benchmark may import
this package.

The paper states the 4:1 ratio and the concatenation with text tokens, not the operator; the reading taken is
the usual patch merger: every `merge` = 4 consecutive visual tokens of a sample are concatenated feature-wise
into one row [merge * d_vit], an MLP projector (linear + bias, exact-erf GELU, linear + bias) maps it to the
LLM width, and the result is written into the LLM's packed embedding stream at that sample's image positions
(the text rows of the stream come from the embedding table).  fp64 throughout; `rnd` rounds where the library
stores a tensor in its storage type."""
import numpy as np

from .ops import gelu_bwd, gelu_fwd, linear_bwd, linear_fwd


def merger_forward(h_vit, w1, b1, w2, b2, positions, x_llm, merge=4, rnd=lambda x: x):
    """h_vit [merge * G, d_vit] -> rows `positions` [G] of x_llm [N_llm, d_llm] (a copy is returned).
    Returns (x_llm_out, cache)."""
    g = h_vit.shape[0] // merge
    assert h_vit.shape[0] == g * merge and len(positions) == g
    cat = h_vit.reshape(g, merge * h_vit.shape[1])           # neighbours are adjacent rows: a pure reshape
    a1 = rnd(linear_fwd(cat, w1, b1))
    act = rnd(gelu_fwd(a1))
    out = rnd(linear_fwd(act, w2, b2))
    x = np.array(x_llm, dtype=np.float64, copy=True)
    x[np.asarray(positions)] = out
    return x, dict(cat=cat, a1=a1, act=act)


def merger_backward(d_x_llm, cache, w1, w2, positions, merge=4, rnd=lambda x: x):
    """Gradient of the rows at `positions` back to the encoder output.  Returns (d_h_vit, dict of weight grads)."""
    d_out = rnd(np.asarray(d_x_llm, dtype=np.float64)[np.asarray(positions)])
    d_act, dw2, db2 = linear_bwd(d_out, cache["act"], w2, True)
    d_a1 = rnd(gelu_bwd(rnd(d_act), cache["a1"]))
    d_cat, dw1, db1 = linear_bwd(d_a1, cache["cat"], w1, True)
    d_h = rnd(d_cat).reshape(-1, cache["cat"].shape[1] // merge)
    return d_h, dict(w1=dw1, b1=db1, w2=dw2, b2=db2)
