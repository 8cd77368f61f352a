"""The layers of the paper's network other than the convolutions (arXiv 1712.02546,
Section 4.1: normalisation, pooling with stride 2, fully connected layer, softmax loss) --
TEST INFRASTRUCTURE.  Plain numpy in float64, written from the textbook definitions; no code
shared with the library; only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may use it.

The paper names the layers and nothing else.  Readings taken here:
  * normalisation = local response normalisation across channels,
        y[n,c,h,w] = x[n,c,h,w] * (kappa + alpha * sum_{c' in W(c)} x[n,c',h,w]^2) ** (-beta),
    W(c) = the `size` channels centred on c (size odd), clipped at the ends;
  * pooling = max pooling over `win` x `win` windows with stride `stride` (the paper: stride 2),
    output extent floor((H - win) / stride) + 1, no padding; the gradient of a window goes to
    its first maximum in row-major order;
  * fully connected: y[n,o] = sum_i x[n,i] * W[o,i] + b[o];
  * softmax loss: mean over the batch of -log softmax(z[n])[label[n]].
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ---- normalisation -----------------------------------------------------------------------
def _window(c: int, C: int, size: int):
    half = size // 2
    return max(0, c - half), min(C, c + half + 1)


def norm_scale(x, size, kappa, alpha):
    """s[n,c,h,w] = kappa + alpha * sum of squares over the channel window of c."""
    x = _f64(x)
    C = x.shape[1]
    s = np.empty_like(x)
    for c in range(C):
        lo, hi = _window(c, C, size)
        s[:, c] = kappa + alpha * np.sum(x[:, lo:hi] ** 2, axis=1)
    return s


def norm_fwd(x, size=5, kappa=1.0, alpha=1e-4, beta=0.75):
    x = _f64(x)
    return x * norm_scale(x, size, kappa, alpha) ** (-beta)


def norm_bwd(x, dy, size=5, kappa=1.0, alpha=1e-4, beta=0.75):
    """dx[c] = dy[c] * s[c]^-beta  -  2*alpha*beta * x[c] * sum_{c' : c in W(c')} dy[c'] * x[c'] * s[c']^(-beta-1)."""
    x, dy = _f64(x), _f64(dy)
    C = x.shape[1]
    s = norm_scale(x, size, kappa, alpha)
    dx = dy * s ** (-beta)
    t = dy * x * s ** (-beta - 1.0)
    for c in range(C):
        # channels c' whose window contains c are exactly the window of c (the window is symmetric)
        lo, hi = _window(c, C, size)
        dx[:, c] -= 2.0 * alpha * beta * x[:, c] * np.sum(t[:, lo:hi], axis=1)
    return dx


# ---- max pooling -------------------------------------------------------------------------
def pool_out(H, win, stride):
    return (H - win) // stride + 1


def pool_fwd(x, win=2, stride=2):
    x = _f64(x)
    N, C, H, W = x.shape
    P, Q = pool_out(H, win, stride), pool_out(W, win, stride)
    y = np.empty((N, C, P, Q))
    for p in range(P):
        for q in range(Q):
            y[:, :, p, q] = x[:, :, p * stride:p * stride + win, q * stride:q * stride + win].max(axis=(2, 3))
    return y


def pool_bwd(x, dy, win=2, stride=2):
    x, dy = _f64(x), _f64(dy)
    N, C, H, W = x.shape
    P, Q = pool_out(H, win, stride), pool_out(W, win, stride)
    dx = np.zeros_like(x)
    for p in range(P):
        for q in range(Q):
            patch = x[:, :, p * stride:p * stride + win, q * stride:q * stride + win].reshape(N, C, win * win)
            arg = np.argmax(patch, axis=2)            # first maximum in row-major order
            i, j = arg // win, arg % win
            n_idx, c_idx = np.meshgrid(np.arange(N), np.arange(C), indexing="ij")
            np.add.at(dx, (n_idx, c_idx, p * stride + i, q * stride + j), dy[:, :, p, q])
    return dx


# ---- fully connected ---------------------------------------------------------------------
def fc_fwd(x, W, b):
    x, W, b = _f64(x), _f64(W), _f64(b)
    return np.einsum("ni,oi->no", x.reshape(x.shape[0], -1), W) + b[None, :]


def fc_bwd(x, W, dy):
    """Returns (dx, dW, db)."""
    x, W, dy = _f64(x), _f64(W), _f64(dy)
    x2 = x.reshape(x.shape[0], -1)
    dx = np.einsum("no,oi->ni", dy, W).reshape(x.shape)
    dW = np.einsum("no,ni->oi", dy, x2)
    db = dy.sum(axis=0)
    return dx, dW, db


# ---- softmax loss ------------------------------------------------------------------------
def softmax(z):
    z = _f64(z)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def softmax_loss_fwd(z, labels):
    p = softmax(z)
    n = np.arange(p.shape[0])
    return float(-np.mean(np.log(p[n, np.asarray(labels)])))


def softmax_loss_bwd(z, labels):
    p = softmax(z)
    n = np.arange(p.shape[0])
    p[n, np.asarray(labels)] -= 1.0
    return p / p.shape[0]


# ---- plain SGD step (the paper trains; no momentum or decay is stated) --------------------
def sgd_update(w, dw, lr):
    return _f64(w) - lr * _f64(dw)
