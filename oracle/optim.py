"""Per-model parameter updates of the oracle (fp64 arithmetic, fp32 storage).

SGD (the optimizer the paper names in passing; Introduction, paragraph on data
parallelism):   p <- p - lr * g, no momentum, no weight decay.
Adam (Kingma & Ba 2015, Algorithm 1, with bias correction):
   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
   p <- p - lr_t * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps),   t = 1, 2, ...
Learning-rate warm-up: lr_t = lr * min(1, t / warmup) when warmup > 0, else lr.
Test infrastructure only.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
OPT_SGD, OPT_ADAM = 0, 1


def lr_at(hp, t: int) -> float:
    """Learning rate of step t (1-based)."""
    w = hp["warmup_steps"]
    return hp["lr"] * min(1.0, t / w) if w > 0 else hp["lr"]


def new_state(params):
    return dict(m=[np.zeros_like(p) for p in params], v=[np.zeros_like(p) for p in params])


def update_tensor(hp, t: int, p, g, m, v):
    """Updates p (and m, v for Adam) in place for step t given the fp64 gradient g."""
    lr = lr_at(hp, t)
    p64 = p.astype(F64)
    if hp["opt"] == OPT_SGD:
        p[...] = (p64 - lr * g).astype(np.float32)
        return
    b1, b2, eps = hp["beta1"], hp["beta2"], hp["eps"]
    m64 = b1 * m.astype(F64) + (1.0 - b1) * g
    v64 = b2 * v.astype(F64) + (1.0 - b2) * g * g
    mhat = m64 / (1.0 - b1 ** t)
    vhat = v64 / (1.0 - b2 ** t)
    p[...] = (p64 - lr * mhat / (np.sqrt(vhat) + eps)).astype(np.float32)
    m[...] = m64.astype(np.float32)
    v[...] = v64.astype(np.float32)
