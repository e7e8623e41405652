"""Float64 definitions of the layer operations (oracle side, test infrastructure).

Each function is the textbook definition written out with one library matrix
product per contraction; nothing is blocked, fused or reordered.  The paper
treats the forward and backward passes as the usual ones (Sec. 1, "first a
forward pass ... following this, a backward pass"); these are those passes.
"""
from __future__ import annotations

import numpy as np


def linear_fwd(x, w, b):
    """z[i, n] = sum_k x[i, k] * w[n, k] + b[n]."""
    return x @ w.T + b


def linear_bwd(dz, x, w, need_dx):
    """dw[n, k] = sum_i dz[i, n] x[i, k]; db[n] = sum_i dz[i, n]; dx[i, k] = sum_n dz[i, n] w[n, k]."""
    dw = dz.T @ x
    db = dz.sum(axis=0)
    dx = dz @ w if need_dx else None
    return dw, db, dx


def relu_fwd(z):
    return np.maximum(z, 0.0)


def relu_bwd(da, z):
    """Derivative taken as 0 at z == 0."""
    return da * (z > 0.0)


def softmax_ce(z, labels):
    """Mean softmax cross-entropy over the rows of z, and its gradient.

    lse_i = m_i + log sum_j exp(z_ij - m_i);  loss = mean_i (lse_i - z_{i, y_i});
    dz_ij = (exp(z_ij - lse_i) - [j == y_i]) / rows.
    """
    rows = z.shape[0]
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    picked = z[np.arange(rows), labels]
    loss = float(np.mean(lse[:, 0] - picked))
    dz = np.exp(z - lse)
    dz[np.arange(rows), labels] -= 1.0
    return loss, dz / rows
