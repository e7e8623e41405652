"""Float64 definitions of the layer operations (oracle side, test infrastructure).

Each function is the textbook definition written out with one library matrix
product per contraction; nothing is blocked, fused or reordered.  The paper
treats the forward and backward passes as the usual ones (Sec. 1: a forward
pass to the loss, then a backward pass for the gradients); these are those passes.
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


# ---- convolutional operations (activations NHWC, weights [Cout, R, S, Cin]) ------------------------

def _pad_hw(x, pad):
    return np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))


def conv_out_size(size, kernel, stride, pad):
    return (size + 2 * pad - kernel) // stride + 1


def conv_fwd(x, w, stride, pad):
    """y[n, ho, wo, co] = sum_{r, t, ci} x[n, ho*stride + r - pad, wo*stride + t - pad, ci] * w[co, r, t, ci], zeros outside x."""
    n, h, wd, _ = x.shape
    co, kr, ks, _ = w.shape
    ho, wo = conv_out_size(h, kr, stride, pad), conv_out_size(wd, ks, stride, pad)
    xp = _pad_hw(x, pad)
    y = np.zeros((n, ho, wo, co))
    for r in range(kr):
        for t in range(ks):
            y += xp[:, r:r + (ho - 1) * stride + 1:stride, t:t + (wo - 1) * stride + 1:stride, :] @ w[:, r, t, :].T
    return y


def conv_wgrad(x, dy, kernel, stride, pad):
    """dw[co, r, t, ci] = sum_{n, ho, wo} dy[n, ho, wo, co] * x[n, ho*stride + r - pad, wo*stride + t - pad, ci]."""
    _, ho, wo, co = dy.shape
    ci = x.shape[3]
    xp = _pad_hw(x, pad)
    dw = np.zeros((co, kernel, kernel, ci))
    flat_dy = dy.reshape(-1, co)
    for r in range(kernel):
        for t in range(kernel):
            patch = xp[:, r:r + (ho - 1) * stride + 1:stride, t:t + (wo - 1) * stride + 1:stride, :]
            dw[:, r, t, :] = flat_dy.T @ patch.reshape(-1, ci)
    return dw


def conv_dgrad(dy, w, in_hw, stride, pad):
    """dx[n, h, wd, ci] = sum over every (ho, wo, r, t, co) whose input position is (h, wd) of dy[n, ho, wo, co] * w[co, r, t, ci]."""
    n, ho, wo, _ = dy.shape
    _, kr, ks, ci = w.shape
    h, wd = in_hw
    dxp = np.zeros((n, h + 2 * pad, wd + 2 * pad, ci))
    for r in range(kr):
        for t in range(ks):
            dxp[:, r:r + (ho - 1) * stride + 1:stride, t:t + (wo - 1) * stride + 1:stride, :] += dy @ w[:, r, t, :]
    return dxp[:, pad:pad + h, pad:pad + wd, :]


def affine_fwd(y, scale, shift):
    """z = scale_c * y + shift_c per channel (a BatchNorm folded to its affine part, kept trainable)."""
    return y * scale + shift


def affine_bwd(dz, y, scale):
    """dscale_c = sum dz * y; dshift_c = sum dz; dy = scale_c * dz."""
    axes = tuple(range(dz.ndim - 1))
    return dz * scale, (dz * y).sum(axis=axes), dz.sum(axis=axes)


def maxpool3x3s2_fwd(x):
    """3x3 window, stride 2, padding 1 acting as -inf.  Returns the output and, per output, the flat input
    position of its maximum (first maximum in row-major window order)."""
    n, h, w, c = x.shape
    ho, wo = conv_out_size(h, 3, 2, 1), conv_out_size(w, 3, 2, 1)
    xp = np.full((n, h + 2, w + 2, c), -np.inf)
    xp[:, 1:h + 1, 1:w + 1, :] = x
    best = np.full((n, ho, wo, c), -np.inf)
    arg = np.zeros((n, ho, wo, c), dtype=np.int64)
    rows = (np.arange(ho) * 2)[None, :, None, None]
    cols = (np.arange(wo) * 2)[None, None, :, None]
    for r in range(3):
        for t in range(3):
            cand = xp[:, r:r + (ho - 1) * 2 + 1:2, t:t + (wo - 1) * 2 + 1:2, :]
            better = cand > best                       # strict: the first maximum wins a tie
            best = np.where(better, cand, best)
            pos = (rows + r - 1) * w + (cols + t - 1)   # flat (h, w) position in the unpadded input
            arg = np.where(better, pos, arg)
    return best, arg


def maxpool3x3s2_bwd(dout, arg, in_hw):
    """Each output's gradient goes to the input position that held its maximum; overlapping windows add."""
    n, ho, wo, c = dout.shape
    h, w = in_hw
    dx = np.zeros((n, h * w, c))
    ni = np.arange(n)[:, None, None, None]
    ci = np.arange(c)[None, None, None, :]
    np.add.at(dx, (ni, arg, ci), dout)
    return dx.reshape(n, h, w, c)


def avgpool_fwd(x):
    return x.mean(axis=(1, 2))


def avgpool_bwd(dp, hw):
    h, w = hw
    return np.broadcast_to(dp[:, None, None, :] / (h * w), (dp.shape[0], h, w, dp.shape[1])).copy()
