"""Oracle for the mini-batch tail of one stage: gradient statistics and one Adam step.

Test infrastructure only (imported by tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg); it shares no code with the HIP path.  Plain numpy, fp64.

What it follows.  The paper keeps, per parameter, 16 bytes of state: a 16-bit parameter and
gradient plus fp32 master weight, momentum and variance (Background, "Memory optimization"),
i.e. mixed-precision Adam; and it synchronises an overflow flag / global gradient norm across
the stages of a pipeline (Enabling Ease of Programming, "Tracking cross-partition
dependencies"; Implementation, "Synchronization of shared state").  One GPU's share of that
is: the sum of squares and the non-finite count of its own accumulated gradients, and the Adam
update of its own parameters.  The update itself is Adam as published (Kingma & Ba,
Algorithm 1) with optional decoupled weight decay; the paper does not restate it.
"""
from __future__ import annotations

import numpy as np


def grad_stats(grads):
    """(sum of squares of all finite entries, number of non-finite entries) over a list of arrays."""
    sumsq, bad = 0.0, 0
    for g in grads:
        g = np.asarray(g, dtype=np.float64).ravel()
        fin = np.isfinite(g)
        bad += int(g.size - fin.sum())
        sumsq += float(np.sum(np.square(g[fin])))
    return sumsq, bad


def adam_step(w, m, v, g, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0):
    """One Adam update, all fp64. step >= 1 is the number of this update (bias correction).
      g' = grad_scale * g
      m  = beta1 m + (1 - beta1) g' ;  v = beta2 v + (1 - beta2) g'^2
      mhat = m / (1 - beta1^step)   ;  vhat = v / (1 - beta2^step)
      w  = w - lr * (mhat / (sqrt(vhat) + eps) + weight_decay * w)
    Returns (w, m, v)."""
    w = np.asarray(w, dtype=np.float64)
    gs = grad_scale * np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * gs
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * gs * gs
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    w = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w, m, v
