"""Sparse update of learnable feature tables with Adam.  TEST INFRASTRUCTURE ONLY.

The paper keeps learnable vectors for featureless node types, updates them after
backpropagation together with their optimizer states, and names Adam's moment and variance
as those states (Sections 2.2 and 6).  Only the rows a mini-batch touched are updated; the
step follows Algorithm 1 of the Adam paper (Kingma & Ba) in its notation, on those rows,
with one global step counter t:

    m <- b1 m + (1 - b1) g            v <- b2 v + (1 - b2) g^2
    mhat = m / (1 - b1^t)             vhat = v / (1 - b2^t)
    theta <- theta - lr * mhat / (sqrt(vhat) + eps)

Everything in fp64; rows not listed in `ids` keep their parameters and their states.
"""
from __future__ import annotations

import numpy as np


def sparse_adam_step(theta: np.ndarray, m: np.ndarray, v: np.ndarray, ids: np.ndarray, grad: np.ndarray,
                     lr: float, beta1: float, beta2: float, eps: float, t: int):
    """Returns (theta, m, v) after step t (t >= 1) as new fp64 arrays; `ids` are distinct rows,
    `grad[i]` is the gradient of row ids[i]."""
    theta = np.array(theta, dtype=np.float64)
    m = np.array(m, dtype=np.float64)
    v = np.array(v, dtype=np.float64)
    ids = np.asarray(ids, dtype=np.int64)
    assert ids.size == np.unique(ids).size, "ids must be distinct"
    assert t >= 1
    for i in range(ids.size):
        r = int(ids[i])
        g = np.asarray(grad[i], dtype=np.float64)
        m[r] = beta1 * m[r] + (1.0 - beta1) * g
        v[r] = beta2 * v[r] + (1.0 - beta2) * g * g
        mhat = m[r] / (1.0 - beta1 ** t)
        vhat = v[r] / (1.0 - beta2 ** t)
        theta[r] = theta[r] - lr * mhat / (np.sqrt(vhat) + eps)
    return theta, m, v
