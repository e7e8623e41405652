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


# ---- Transformer encoder operations --------------------------------------------------------------

LN_EPS = 1e-5


def layernorm_fwd(x, gamma, beta):
    """Per row: mu = mean(x), var = mean((x - mu)^2) (biased), xhat = (x - mu) / sqrt(var + eps), y = gamma * xhat + beta."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def layernorm_bwd(dy, gamma, cache):
    """g = dy * gamma; dx = (g - mean(g) - xhat * mean(g * xhat)) * rstd; dgamma = sum_rows dy * xhat; dbeta = sum_rows dy."""
    xhat, rstd = cache
    g = dy * gamma
    dx = (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True)) * rstd
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def _erf(x):
    from scipy.special import erf
    return erf(x)


def gelu_fwd(x):
    """Exact GELU: x * Phi(x) with the normal distribution function Phi(x) = (1 + erf(x / sqrt 2)) / 2."""
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x), phi the normal density."""
    return 0.5 * (1.0 + _erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)


def softmax_rows(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def split_heads(t, batch, seq, heads):
    """[batch * seq, heads * d] -> [batch, heads, seq, d]."""
    d = t.shape[1] // heads
    return t.reshape(batch, seq, heads, d).transpose(0, 2, 1, 3)


def merge_heads(t):
    """[batch, heads, seq, d] -> [batch * seq, heads * d]."""
    b, h, s, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b * s, h * d)
