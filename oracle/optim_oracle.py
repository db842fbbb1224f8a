"""CPU oracle of the adapter update (TEST INFRASTRUCTURE; Harli Sec. 2.1: finetuning = forward, backward, update).

The paper names no optimizer; the reading taken is AdamW with decoupled weight decay (the default of the
finetuning framework it builds on), written out in NumPy float64:

    m <- b1*m + (1-b1)*g          v <- b2*v + (1-b2)*g*g
    p <- p - lr * ( (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps) + wd * p )        t = 1, 2, ...

`grad_scale` multiplies g first (gradient accumulation / loss scaling).  Parameters, moments and the result are
float64 here; the library keeps fp32 master parameters and moments and writes a bf16 copy for the kernels.
"""
from __future__ import annotations

import numpy as np


def adamw_step(p, g, m, v, t, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8, wd=0.0, grad_scale=1.0):
    p, g, m, v = (np.asarray(a, np.float64) for a in (p, g, m, v))
    g = g * grad_scale
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + wd * p)
    return p, m, v
