"""Layer definitions for the step oracle, fp64 numpy, channels-last (test infrastructure).

Each forward is the textbook definition of the operation written out directly;
each backward is its derivative.  A matrix product from numpy serves as a
step; there is no tiling, fusion or reordering.  These are the inner
function F of the per-worker gradient in Algorithm 1 (the gradient line of
procedure Train) for the benchmark networks.
"""
from __future__ import annotations

import numpy as np


# ---------------------------------------------------------------- linear
def linear_fwd(x, W, b):
    """x [n, cin], W [cout, cin], b [cout] or None -> [n, cout]."""
    y = x @ W.T
    if b is not None:
        y = y + b
    return y


def linear_bwd(x, W, dy):
    dx = dy @ W
    dW = dy.T @ x
    db = dy.sum(axis=0)
    return dx, dW, db


# ---------------------------------------------------------------- convolution
def conv_fwd(x, W, b, stride, pad):
    """x [n, H, W, cin], W [cout, kh, kw, cin] -> [n, Ho, Wo, cout]:
    y[n,i,j,o] = b[o] + sum_{u,v,c} x[n, i*stride+u-pad, j*stride+v-pad, c] * W[o,u,v,c]
    with zeros outside the image."""
    n, H, Wd, cin = x.shape
    cout, kh, kw, _ = W.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    xp = np.zeros((n, H + 2 * pad, Wd + 2 * pad, cin), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + Wd, :] = x
    y = np.zeros((n, Ho, Wo, cout), dtype=np.float64)
    for u in range(kh):
        for v in range(kw):
            patch = xp[:, u:u + stride * Ho:stride, v:v + stride * Wo:stride, :]
            y += patch @ W[:, u, v, :].T
    if b is not None:
        y = y + b
    return y


def conv_bwd(x, W, dy, stride, pad):
    n, H, Wd, cin = x.shape
    cout, kh, kw, _ = W.shape
    _, Ho, Wo, _ = dy.shape
    xp = np.zeros((n, H + 2 * pad, Wd + 2 * pad, cin), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + Wd, :] = x
    dxp = np.zeros_like(xp)
    dW = np.zeros_like(W, dtype=np.float64)
    dy2 = dy.reshape(-1, cout)
    for u in range(kh):
        for v in range(kw):
            patch = xp[:, u:u + stride * Ho:stride, v:v + stride * Wo:stride, :]
            dW[:, u, v, :] = dy2.T @ patch.reshape(-1, cin)
            dxp[:, u:u + stride * Ho:stride, v:v + stride * Wo:stride, :] += dy @ W[:, u, v, :]
    dx = dxp[:, pad:pad + H, pad:pad + Wd, :]
    db = dy2.sum(axis=0)
    return dx, dW, db


# ---------------------------------------------------------------- relu
def relu_fwd(x):
    return np.maximum(x, 0.0)


def relu_bwd(x, dy):
    """Derivative 1 where the input is positive, 0 elsewhere (0 at exactly 0)."""
    return dy * (x > 0.0)


# ---------------------------------------------------------------- 2x2 max pool, stride 2
def _windows(x):
    n, H, W, c = x.shape
    w = x.reshape(n, H // 2, 2, W // 2, 2, c).transpose(0, 1, 3, 2, 4, 5)
    return w.reshape(n, H // 2, W // 2, 4, c)      # window entries in (dy, dx) scan order


def maxpool2_fwd(x):
    return _windows(x).max(axis=3)


def maxpool2_bwd(x, dy):
    """The gradient goes to the first maximal entry of each window in (dy, dx) scan order."""
    n, H, W, c = x.shape
    w = _windows(x)
    first = np.argmax(w, axis=3)                    # first occurrence of the maximum
    g = np.zeros_like(w)
    np.put_along_axis(g, first[:, :, :, None, :], dy[:, :, :, None, :], axis=3)
    g = g.reshape(n, H // 2, W // 2, 2, 2, c).transpose(0, 1, 3, 2, 4, 5)
    return g.reshape(n, H, W, c)


# ---------------------------------------------------------------- batch norm (training mode)
BN_EPS = 1e-5


def bn_fwd(x, gamma, beta):
    """Normalise each channel with the mean and biased variance of the rows given
    (one worker's rows): y = gamma * (x - mu) / sqrt(var + eps) + beta."""
    ax = tuple(range(x.ndim - 1))
    mu = x.mean(axis=ax)
    var = ((x - mu) ** 2).mean(axis=ax)
    xhat = (x - mu) / np.sqrt(var + BN_EPS)
    return gamma * xhat + beta, (xhat, var)


def bn_bwd(cache, gamma, dy):
    xhat, var = cache
    ax = tuple(range(dy.ndim - 1))
    dbeta = dy.sum(axis=ax)
    dgamma = (dy * xhat).sum(axis=ax)
    m_dy = dy.mean(axis=ax)
    m_dyx = (dy * xhat).mean(axis=ax)
    dx = gamma / np.sqrt(var + BN_EPS) * (dy - m_dy - xhat * m_dyx)
    return dx, dgamma, dbeta


# ---------------------------------------------------------------- global average pool
def gap_fwd(x):
    return x.mean(axis=(1, 2), keepdims=True)


def gap_bwd(x, dy):
    n, H, W, c = x.shape
    return np.broadcast_to(dy / (H * W), x.shape).copy()


# ---------------------------------------------------------------- softmax cross-entropy
def softmax_xent(z, labels):
    """Per-row loss -log softmax(z)[label] (natural log, max-subtracted) and the
    row-wise derivative softmax(z) - onehot(label), both unscaled."""
    zs = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(zs).sum(axis=1))
    rows = np.arange(z.shape[0])
    loss = lse - zs[rows, labels]
    p = np.exp(zs - lse[:, None])
    p[rows, labels] -= 1.0
    return loss, p


# ---------------------------------------------------------------- bf16 storage model
def round_bf16(a):
    """Round to the nearest bf16 value, ties to even (models a bf16 store of an fp32 result)."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)
