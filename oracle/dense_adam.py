"""Float64 statement of the dense (AllReduce-style) step: weighted average, then Adam.

Test infrastructure: see the package docstring.  Section II notes that the
Parameter-Server formulation carries over to AllReduce by dropping the
server term; what is left on one device is the reduction of the K workers'
gradient buffers (weights B_k / B) and the optimizer step on the result.
The optimizer is Adam with bias correction (Kingma & Ba, Algorithm 1).
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def weighted_average(grads: Sequence[np.ndarray], weights: Sequence[float]) -> np.ndarray:
    """g = sum_k w_k g_k, accumulated in float64 in buffer order."""
    g = np.zeros(np.shape(grads[0]), dtype=np.float64)
    for gk, wk in zip(grads, weights):
        g += float(wk) * np.asarray(gk, dtype=np.float64)
    return g


def adam_step(p, m, v, g, lr, beta1, beta2, eps, step):
    """m' = b1 m + (1-b1) g;  v' = b2 v + (1-b2) g^2;
    p' = p - lr * (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps),  t = step >= 1."""
    p, m, v, g = (np.asarray(a, dtype=np.float64) for a in (p, m, v, g))
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - beta1 ** step)
    vhat = v1 / (1.0 - beta2 ** step)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m1, v1


def dense_aggregate_adam(p, m, v, grads, weights, lr, beta1, beta2, eps, step):
    """Weighted average of the K buffers followed by one Adam step; float64 results."""
    return adam_step(p, m, v, weighted_average(grads, weights), lr, beta1, beta2, eps, step)
