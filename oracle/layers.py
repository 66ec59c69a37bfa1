"""Layer forward / backward passes of the CPU oracle, fp64 numpy, from the definitions.

Test infrastructure (CPU oracle).  Every function takes the weights it should
use as an argument: the backward pass of TiMePReSt differentiates with respect
to the weights as they are when the backward pass runs, while everything that
depends on activations (inputs, ReLU masks, pooling winners, softmax
probabilities) is what the forward pass stored (Methodology, Challenge 1 and
its Solution).  Layouts: dense activations [B, D]; images channels-last
[B, H, W, C]; dense weights [Dout, Din]; filters [Cout, R, S, Cin].
"""
import numpy as np


# ----------------------------------------------------------------------------- linear
def linear_forward(x, w, b, relu):
    """y = x w^T + b, optionally followed by max(., 0).  Returns (y, cache)."""
    x2 = x.reshape(x.shape[0], -1)
    y = x2 @ w.T + b
    if relu:
        y = np.maximum(y, 0.0)
    return y, {"x": x2, "y": y, "x_shape": x.shape}


def linear_backward(dy, cache, w_now, relu):
    """Gradients of a linear(+ReLU) layer.  Returns (dx, dw, db)."""
    dz = dy * (cache["y"] > 0.0) if relu else dy
    dx = dz @ w_now
    dw = dz.T @ cache["x"]
    db = dz.sum(axis=0)
    return dx.reshape(cache["x_shape"]), dw, db


# ----------------------------------------------------------------------------- convolution
def conv_forward(x, w, b, stride, pad, relu):
    """y[n,p,q,o] = b[o] + sum_{r,s,c} xpad[n, p*stride+r, q*stride+s, c] * w[o,r,s,c]."""
    n, h, wd, c = x.shape
    co, R, S, _ = w.shape
    ho = (h + 2 * pad - R) // stride + 1
    wo = (wd + 2 * pad - S) // stride + 1
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), dtype=np.float64)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    y = np.zeros((n, ho, wo, co), dtype=np.float64) + b
    for r in range(R):
        for s in range(S):
            patch = xp[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :]
            y += patch @ w[:, r, s, :].T
    if relu:
        y = np.maximum(y, 0.0)
    return y, {"xp": xp, "y": y, "x_shape": x.shape}


def conv_backward(dy, cache, w_now, stride, pad, relu):
    """Returns (dx, dw, db) of the convolution above."""
    dz = dy * (cache["y"] > 0.0) if relu else dy
    xp = cache["xp"]
    n, h, wd, c = cache["x_shape"]
    co, R, S, _ = w_now.shape
    _, ho, wo, _ = dz.shape
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w_now, dtype=np.float64)
    dz2 = dz.reshape(-1, co)
    for r in range(R):
        for s in range(S):
            patch = xp[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :]
            dw[:, r, s, :] = dz2.T @ patch.reshape(-1, c)
            dxp[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :] += dz @ w_now[:, r, s, :]
    dx = dxp[:, pad:pad + h, pad:pad + wd, :]
    db = dz2.sum(axis=0)
    return dx, dw, db


# ----------------------------------------------------------------------------- max pooling
def maxpool_forward(x, k, stride):
    """Window maximum; the winner of a window is its first maximum in row-major window order."""
    n, h, wd, c = x.shape
    ho = (h - k) // stride + 1
    wo = (wd - k) // stride + 1
    y = np.full((n, ho, wo, c), -np.inf)
    win = np.zeros((n, ho, wo, c), dtype=np.int64)
    for r in range(k):
        for s in range(k):
            v = x[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :]
            better = v > y
            y = np.where(better, v, y)
            win = np.where(better, r * k + s, win)
    return y, {"win": win, "x_shape": x.shape}


def maxpool_backward(dy, cache, k, stride):
    n, h, wd, c = cache["x_shape"]
    _, ho, wo, _ = dy.shape
    dx = np.zeros((n, h, wd, c))
    for r in range(k):
        for s in range(k):
            dx[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :] += dy * (cache["win"] == r * k + s)
    return dx


# ----------------------------------------------------------------------------- loss
def softmax_ce_forward(logits, labels):
    """Mean cross-entropy of a micro-batch and the softmax probabilities."""
    z = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(z)
    ssum = e.sum(axis=1, keepdims=True)
    p = e / ssum
    rows = np.arange(logits.shape[0])
    loss = float(np.mean(np.log(ssum[:, 0]) - z[rows, labels]))
    return loss, {"p": p, "labels": labels}


def softmax_ce_backward(cache, M):
    """Gradient of (1/M) * sum over the mini-batch's M samples of the per-sample loss,
    i.e. of the average of the N equal-sized micro-batch losses (section "Work Scheduling")."""
    p = cache["p"]
    g = p.copy()
    g[np.arange(p.shape[0]), cache["labels"]] -= 1.0
    return g / M
