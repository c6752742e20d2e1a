"""Oracle for the student's parameter update (Sec. 2.2: the student alone runs "optimizer-driven parameter
updates").  TEST INFRASTRUCTURE ONLY: only tests/, the smoke check and the CPU-baseline leg of the benchmark
may import this package.

The paper names no optimizer; the reading taken here is AdamW (Adam with decoupled weight decay, Loshchilov &
Hutter), the usual choice for LLM training, written out from its definition in fp64:

    g   = grad_scale * grad
    m   = beta1 m + (1 - beta1) g
    v   = beta2 v + (1 - beta2) g^2
    w   = w (1 - lr wd) - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)          t = 1, 2, ...

The master weights, m and v are fp32 state; the model's weights are the master weights rounded to the storage
type (`rnd`).  `rnd_state` rounds the state after each update (fp32 in the library)."""
import numpy as np


def adamw_step(w, m, v, grad, step, lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, grad_scale=1.0,
               rnd=lambda x: x, rnd_state=lambda x: x):
    """Returns (w_master, m, v, w_model) after update number `step` (1-based)."""
    w, m, v, g = (np.asarray(a, dtype=np.float64) for a in (w, m, v, grad))
    g = grad_scale * g
    m = rnd_state(beta1 * m + (1.0 - beta1) * g)
    v = rnd_state(beta2 * v + (1.0 - beta2) * g * g)
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    w = rnd_state(w * (1.0 - lr * weight_decay) - lr * m_hat / (np.sqrt(v_hat) + eps))
    return w, m, v, rnd(w)
