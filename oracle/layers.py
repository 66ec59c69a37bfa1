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
from scipy.special import erf


# ----------------------------------------------------------------------------- linear
def gelu(z):
    """Gaussian error linear unit, exact form: z * Phi(z) with Phi the standard normal CDF."""
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_derivative(z):
    """d/dz [z Phi(z)] = Phi(z) + z phi(z)."""
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def linear_forward(x, w, b, relu, act=None, rows=1, skip=None, round_z=None):
    """y = act(x w^T + b) [+ skip].  act: None, "relu" (also relu=True) or "gelu".

    rows: rows per sample; the layer acts on every row of [B, rows, Din] independently.
    skip: tensor added to the result (a residual connection), same shape as y.
    round_z: storage rounding applied to the pre-activation kept for the GELU derivative.
    Returns (y, cache)."""
    x2 = x.reshape(x.shape[0] * rows, -1)
    z = x2 @ w.T + b
    if relu or act == "relu":
        y = np.maximum(z, 0.0)
    elif act == "gelu":
        y = gelu(z)
    else:
        y = z
    if skip is not None:
        y = y + skip.reshape(y.shape)
    y = y.reshape((x.shape[0], -1))
    cache = {"x": x2, "y": y, "x_shape": x.shape}
    if act == "gelu":
        cache["z"] = z if round_z is None else round_z(z)
    return y, cache


def linear_backward(dy, cache, w_now, relu, act=None):
    """Gradients of a linear(+activation) layer w.r.t. input, weight, bias.  Returns (dx, dw, db).
    The gradient of a residual connection (dy itself, towards the skip source) is the caller's."""
    x2 = cache["x"]
    dy2 = dy.reshape(x2.shape[0], -1)
    if relu or act == "relu":
        dz = dy2 * (cache["y"].reshape(dy2.shape) > 0.0)
    elif act == "gelu":
        dz = dy2 * gelu_derivative(cache["z"])
    else:
        dz = dy2
    dx = dz @ w_now
    dw = dz.T @ x2
    db = dz.sum(axis=0)
    return dx.reshape(cache["x_shape"]), dw, db


# ----------------------------------------------------------------------------- layer normalisation
def layernorm_forward(x, gamma, beta, d, eps=1e-5):
    """Per row of d features: y = gamma * (x - mean) / sqrt(var + eps) + beta (biased variance)."""
    x2 = x.reshape(-1, d)
    mean = x2.mean(axis=1, keepdims=True)
    var = ((x2 - mean) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x2 - mean) * rstd
    y = xhat * gamma + beta
    return y.reshape(x.shape), {"xhat": xhat, "rstd": rstd, "x_shape": x.shape}


def layernorm_backward(dy, cache, gamma_now):
    """Returns (dx, dgamma, dbeta).  The normalised input and 1/std are the forward pass's."""
    xhat, rstd = cache["xhat"], cache["rstd"]
    dy2 = dy.reshape(xhat.shape)
    g = dy2 * gamma_now
    dx = rstd * (g - g.mean(axis=1, keepdims=True) - xhat * (g * xhat).mean(axis=1, keepdims=True))
    return dx.reshape(cache["x_shape"]), (dy2 * xhat).sum(axis=0), dy2.sum(axis=0)


# ----------------------------------------------------------------------------- attention
def attention_forward(qkv, s, d, heads):
    """Causal multi-head self-attention on packed [B, s, 3d] = (q | k | v), heads of d/heads features:
    out[b, i, h] = sum_{j <= i} softmax_j(q_i . k_j / sqrt(dh)) v_j."""
    B = qkv.shape[0]
    dh = d // heads
    t = qkv.reshape(B, s, 3, heads, dh)
    q, k, v = (t[:, :, i].transpose(0, 2, 1, 3) for i in range(3))      # [B, heads, s, dh]
    sc = q @ k.transpose(0, 1, 3, 2) / np.sqrt(dh)
    future = np.triu(np.ones((s, s), dtype=bool), 1)
    sc = np.where(future, -np.inf, sc)
    sc = sc - sc.max(axis=-1, keepdims=True)
    e = np.exp(sc)
    p = e / e.sum(axis=-1, keepdims=True)
    o = p @ v
    out = o.transpose(0, 2, 1, 3).reshape(B, s * d)
    return out, {"q": q, "k": k, "v": v, "p": p, "dims": (B, s, d, heads, dh)}


def attention_backward(dy, cache):
    """Gradient w.r.t. the packed qkv input."""
    B, s, d, heads, dh = cache["dims"]
    q, k, v, p = cache["q"], cache["k"], cache["v"], cache["p"]
    do = dy.reshape(B, s, heads, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = ds @ k / np.sqrt(dh)
    dk = ds.transpose(0, 1, 3, 2) @ q / np.sqrt(dh)
    t = np.stack([dq, dk, dv], axis=0).transpose(1, 3, 0, 2, 4)          # [B, s, 3, heads, dh]
    return t.reshape(B, s * 3 * d)


# ----------------------------------------------------------------------------- embedding
def embedding_forward(tokens, wte, wpe):
    """out[b, i] = wte[tokens[b, i]] + wpe[i]."""
    tok = np.asarray(tokens).astype(np.int64)
    B, s = tok.shape
    out = wte[tok] + wpe[None, :s, :]
    return out.reshape(B, -1), {"tok": tok}


def embedding_backward(dy, cache, vocab, d):
    """Returns (dwte, dwpe): rows of dy added onto the token's row / summed over the batch."""
    tok = cache["tok"]
    B, s = tok.shape
    dy3 = dy.reshape(B, s, d)
    dwte = np.zeros((vocab, d))
    np.add.at(dwte, tok.reshape(-1), dy3.reshape(-1, d))
    return dwte, dy3.sum(axis=0)


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


# ----------------------------------------------------------------------------- per-channel affine
def affine_forward(x, gain, shift, relu):
    """y[..., c] = gain[c] * x[..., c] + shift[c], then ReLU if asked (channels last)."""
    y = x * gain + shift
    if relu:
        y = np.maximum(y, 0.0)
    return y, {"x": x, "y": y}


def affine_backward(dy, cache, gain_now, relu):
    """Returns (dx, dgain, dshift); the ReLU mask and the input are the forward pass's."""
    x = cache["x"]
    dz = dy.reshape(x.shape)
    if relu:
        dz = dz * (cache["y"] > 0.0)
    c = x.shape[-1]
    return dz * gain_now, (dz * x).reshape(-1, c).sum(axis=0), dz.reshape(-1, c).sum(axis=0)


# ----------------------------------------------------------------------------- residual join
def resadd_forward(a, b, relu):
    """y = act(a + b)."""
    y = a + b.reshape(a.shape)
    if relu:
        y = np.maximum(y, 0.0)
    return y, {"y": y}


def resadd_backward(dy, cache, relu):
    """Gradient w.r.t. a (and, identically, w.r.t. b)."""
    dz = dy.reshape(cache["y"].shape)
    return dz * (cache["y"] > 0.0) if relu else dz


# ----------------------------------------------------------------------------- global average pooling
def avgpool_forward(x):
    """[B, H, W, C] -> [B, C]: mean over the H*W positions."""
    n, h, wd, c = x.shape
    return x.reshape(n, h * wd, c).mean(axis=1), {"x_shape": x.shape}


def avgpool_backward(dy, cache):
    n, h, wd, c = cache["x_shape"]
    return np.broadcast_to(dy.reshape(n, 1, 1, c) / (h * wd), (n, h, wd, c)).copy()


# ----------------------------------------------------------------------------- max pooling
def maxpool_forward(x, k, stride, pad=0):
    """Window maximum; the winner of a window is its first maximum in row-major window order.
    pad: rows / columns of padding on every side, which never win (they count as -infinity)."""
    n, h, wd, c = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    xp = np.full((n, h + 2 * pad, wd + 2 * pad, c), -np.inf)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    y = np.full((n, ho, wo, c), -np.inf)
    win = np.zeros((n, ho, wo, c), dtype=np.int64)
    for r in range(k):
        for s in range(k):
            v = xp[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :]
            better = v > y
            y = np.where(better, v, y)
            win = np.where(better, r * k + s, win)
    return y, {"win": win, "x_shape": x.shape}


def maxpool_backward(dy, cache, k, stride, pad=0):
    n, h, wd, c = cache["x_shape"]
    _, ho, wo, _ = dy.shape
    dxp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c))
    for r in range(k):
        for s in range(k):
            dxp[:, r:r + stride * ho:stride, s:s + stride * wo:stride, :] += dy * (cache["win"] == r * k + s)
    return dxp[:, pad:pad + h, pad:pad + wd, :]


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
