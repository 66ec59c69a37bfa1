"""Pins of the oracle's layer arithmetic: closed forms, finite differences, library autograd."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L

torch.set_default_dtype(torch.float64)


def _fd(f, x, eps=1e-6):
    """Central finite-difference gradient of scalar f at x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f()
        x[i] = old - eps
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def _rel(a, b):
    return np.max(np.abs(a - b)) / (np.max(np.abs(b)) + 1e-300)


# ------------------------------------------------------------------ softmax cross-entropy
def test_ce_uniform_logits_closed_form():
    C, B, M = 10, 6, 24
    labels = np.arange(B) % C
    loss, c = L.softmax_ce_forward(np.full((B, C), 3.7), labels)
    assert abs(loss - np.log(C)) < 1e-14
    g = L.softmax_ce_backward(c, M)
    want = np.full((B, C), 1.0 / C)
    want[np.arange(B), labels] -= 1.0
    assert np.allclose(g, want / M, atol=1e-16)


def test_ce_rows_sum_to_zero_and_shift_invariance():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((5, 7)) * 4
    y = rng.integers(0, 7, 5)
    l1, c1 = L.softmax_ce_forward(z, y)
    l2, c2 = L.softmax_ce_forward(z + 1000.0, y)
    assert abs(l1 - l2) < 1e-9
    assert np.allclose(L.softmax_ce_backward(c1, 5).sum(axis=1), 0.0, atol=1e-15)


def test_ce_against_library_and_finite_differences():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((8, 10))
    y = rng.integers(0, 10, 8)
    loss, c = L.softmax_ce_forward(z, y)
    zt = torch.tensor(z, requires_grad=True)
    lt = F.cross_entropy(zt, torch.tensor(y))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    # gradient of the mean over these 8 rows == softmax_ce_backward with M = 8
    assert _rel(L.softmax_ce_backward(c, 8), zt.grad.numpy()) < 1e-12
    g_fd = _fd(lambda: L.softmax_ce_forward(z, y)[0], z)
    assert _rel(L.softmax_ce_backward(c, 8), g_fd) < 1e-7
    # a mini-batch of M = 32 of which this is one micro-batch: gradient scales by 8/32
    assert np.allclose(L.softmax_ce_backward(c, 32) * 4, L.softmax_ce_backward(c, 8))


# ------------------------------------------------------------------ linear
@pytest.mark.parametrize("relu", [False, True])
def test_linear_against_library_autograd(relu):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 7)); w = rng.standard_normal((4, 7)); b = rng.standard_normal(4)
    dy = rng.standard_normal((5, 4))
    y, c = L.linear_forward(x, w, b, relu)
    dx, dw, db = L.linear_backward(dy, c, w, relu)
    xt, wt, bt = (torch.tensor(a, requires_grad=True) for a in (x, w, b))
    yt = F.linear(xt, wt, bt)
    if relu:
        yt = F.relu(yt)
    yt.backward(torch.tensor(dy))
    assert _rel(y, yt.detach().numpy()) < 1e-13
    assert _rel(dx, xt.grad.numpy()) < 1e-13
    assert _rel(dw, wt.grad.numpy()) < 1e-13
    assert _rel(db, bt.grad.numpy()) < 1e-13


def test_linear_finite_differences():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 5)); w = rng.standard_normal((4, 5)); b = rng.standard_normal(4)
    r = rng.standard_normal((3, 4))
    f = lambda: float((L.linear_forward(x, w, b, True)[0] * r).sum())
    y, c = L.linear_forward(x, w, b, True)
    dx, dw, db = L.linear_backward(r, c, w, True)
    assert _rel(dx, _fd(f, x)) < 1e-7
    assert _rel(dw, _fd(f, w)) < 1e-7
    assert _rel(db, _fd(f, b)) < 1e-7


def test_linear_backward_uses_the_weights_it_is_given():
    # dx must come from the weights passed to backward, dw and the mask from the stored forward
    rng = np.random.default_rng(4)
    x = rng.standard_normal((3, 5)); w0 = rng.standard_normal((4, 5)); w1 = rng.standard_normal((4, 5))
    b = rng.standard_normal(4); dy = rng.standard_normal((3, 4))
    y, c = L.linear_forward(x, w0, b, True)
    dx, dw, db = L.linear_backward(dy, c, w1, True)
    dz = dy * (x @ w0.T + b > 0)
    assert np.allclose(dx, dz @ w1)
    assert np.allclose(dw, dz.T @ x)


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("R,stride,pad,relu", [(3, 1, 1, True), (3, 1, 1, False), (1, 1, 0, False),
                                               (3, 2, 1, True), (1, 2, 0, False), (7, 2, 3, True)])
def test_conv_against_library_autograd(R, stride, pad, relu):
    rng = np.random.default_rng(5)
    n, h, wd, ci, co = 2, 9, 8, 3, 4
    x = rng.standard_normal((n, h, wd, ci)); w = rng.standard_normal((co, R, R, ci)); b = rng.standard_normal(co)
    y, c = L.conv_forward(x, w, b, stride, pad, relu)
    dy = rng.standard_normal(y.shape)
    dx, dw, db = L.conv_backward(dy, c, w, stride, pad, relu)
    xt = torch.tensor(x.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    wt = torch.tensor(w.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    yt = F.conv2d(xt, wt, bt, stride=stride, padding=pad)
    if relu:
        yt = F.relu(yt)
    yt.backward(torch.tensor(dy.transpose(0, 3, 1, 2).copy()))
    assert y.shape == tuple(yt.permute(0, 2, 3, 1).shape)
    assert _rel(y, yt.detach().permute(0, 2, 3, 1).numpy()) < 1e-12
    assert _rel(dx, xt.grad.permute(0, 2, 3, 1).numpy()) < 1e-12
    assert _rel(dw, wt.grad.permute(0, 2, 3, 1).numpy()) < 1e-12
    assert _rel(db, bt.grad.numpy()) < 1e-12


def test_conv_brute_force_tiny():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((1, 4, 5, 2)); w = rng.standard_normal((3, 3, 3, 2)); b = rng.standard_normal(3)
    y, _ = L.conv_forward(x, w, b, 1, 1, False)
    for p in range(4):
        for q in range(5):
            for o in range(3):
                acc = b[o]
                for r in range(3):
                    for s in range(3):
                        hh, ww = p + r - 1, q + s - 1
                        if 0 <= hh < 4 and 0 <= ww < 5:
                            for ch in range(2):
                                acc += x[0, hh, ww, ch] * w[o, r, s, ch]
                assert abs(acc - y[0, p, q, o]) < 1e-12


def test_conv_1x1_is_a_linear_layer():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 3, 3, 5)); w = rng.standard_normal((4, 1, 1, 5)); b = rng.standard_normal(4)
    y, _ = L.conv_forward(x, w, b, 1, 0, True)
    y2, _ = L.linear_forward(x.reshape(-1, 5), w.reshape(4, 5), b, True)
    assert np.allclose(y.reshape(-1, 4), y2)


# ------------------------------------------------------------------ max pooling
@pytest.mark.parametrize("k,stride", [(2, 2), (3, 2)])
def test_maxpool_against_library_autograd(k, stride):
    rng = np.random.default_rng(8)
    x = rng.standard_normal((2, 8, 9, 3))
    y, c = L.maxpool_forward(x, k, stride)
    dy = rng.standard_normal(y.shape)
    dx = L.maxpool_backward(dy, c, k, stride)
    xt = torch.tensor(x.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    yt = F.max_pool2d(xt, k, stride)
    yt.backward(torch.tensor(dy.transpose(0, 3, 1, 2).copy()))
    assert np.array_equal(y, yt.detach().permute(0, 2, 3, 1).numpy())
    assert np.allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy())


def test_maxpool_gradient_goes_to_one_winner_per_window():
    x = np.zeros((1, 2, 2, 1)); x[0, 1, 0, 0] = 2.0
    y, c = L.maxpool_forward(x, 2, 2)
    dx = L.maxpool_backward(np.ones_like(y), c, 2, 2)
    assert y[0, 0, 0, 0] == 2.0 and dx[0, 1, 0, 0] == 1.0 and dx.sum() == 1.0
    # all-equal window: exactly one element (the first) receives the gradient
    y, c = L.maxpool_forward(np.zeros((1, 2, 2, 1)), 2, 2)
    dx = L.maxpool_backward(np.ones_like(y), c, 2, 2)
    assert dx.sum() == 1.0 and dx[0, 0, 0, 0] == 1.0


@pytest.mark.parametrize("k,stride,pad", [(3, 2, 1), (2, 2, 1)])
def test_padded_maxpool_against_library_autograd(k, stride, pad):
    rng = np.random.default_rng(18)
    x = rng.standard_normal((2, 9, 8, 3)) - 2.0   # mostly negative: padding (which never wins) must not read as 0
    y, c = L.maxpool_forward(x, k, stride, pad)
    dy = rng.standard_normal(y.shape)
    dx = L.maxpool_backward(dy, c, k, stride, pad)
    xt = torch.tensor(x.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    yt = F.max_pool2d(xt, k, stride, padding=pad)
    yt.backward(torch.tensor(dy.transpose(0, 3, 1, 2).copy()))
    assert np.array_equal(y, yt.detach().permute(0, 2, 3, 1).numpy())
    assert np.allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy())


# ------------------------------------------------------------------ per-channel affine, residual join, average pooling
@pytest.mark.parametrize("relu", [False, True])
def test_affine_against_library_autograd_and_fd(relu):
    rng = np.random.default_rng(19)
    x = rng.standard_normal((3, 4, 5, 6))
    g = rng.standard_normal(6) + 1.0
    b = rng.standard_normal(6)
    y, c = L.affine_forward(x, g, b, relu)
    dy = rng.standard_normal(y.shape)
    dx, dg, db = L.affine_backward(dy, c, g, relu)
    xt, gt, bt = (torch.tensor(v, requires_grad=True) for v in (x, g, b))
    yt = xt * gt + bt
    if relu:
        yt = F.relu(yt)
    yt.backward(torch.tensor(dy))
    assert np.allclose(y, yt.detach().numpy()) and np.allclose(dx, xt.grad.numpy())
    assert np.allclose(dg, gt.grad.numpy()) and np.allclose(db, bt.grad.numpy())
    # the same layer is what a batch-normalisation layer computes at inference with mean 0 and variance 1 - eps
    bn = F.batch_norm(torch.tensor(x).permute(0, 3, 1, 2), torch.zeros(6), torch.ones(6) - 1e-5, torch.tensor(g),
                      torch.tensor(b), training=False, eps=1e-5).permute(0, 2, 3, 1)
    assert np.allclose(np.maximum(bn.numpy(), 0.0) if relu else bn.numpy(), y)
    # finite differences of sum(dy * y) w.r.t. the gain
    f = lambda: float(np.sum(dy * L.affine_forward(x, g, b, relu)[0]))
    assert _rel(_fd(f, g), dg) < 1e-6


def test_affine_backward_uses_the_gain_it_is_given():
    rng = np.random.default_rng(20)
    x = rng.standard_normal((2, 3, 3, 4))
    g0, g1 = rng.standard_normal(4), rng.standard_normal(4)
    y, c = L.affine_forward(x, g0, np.zeros(4), False)
    dy = rng.standard_normal(y.shape)
    assert np.allclose(L.affine_backward(dy, c, g1, False)[0], dy * g1)


@pytest.mark.parametrize("relu", [False, True])
def test_resadd_and_avgpool_against_library(relu):
    rng = np.random.default_rng(21)
    a, b = rng.standard_normal((2, 3, 4, 5)), rng.standard_normal((2, 3, 4, 5))
    y, c = L.resadd_forward(a, b, relu)
    dy = rng.standard_normal(y.shape)
    da = L.resadd_backward(dy, c, relu)
    at, bt = torch.tensor(a, requires_grad=True), torch.tensor(b, requires_grad=True)
    yt = F.relu(at + bt) if relu else at + bt
    yt.backward(torch.tensor(dy))
    assert np.allclose(y, yt.detach().numpy()) and np.allclose(da, at.grad.numpy()) and np.allclose(da, bt.grad.numpy())
    p, c = L.avgpool_forward(a)
    dp = rng.standard_normal(p.shape)
    at = torch.tensor(a.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    pt = F.adaptive_avg_pool2d(at, 1).flatten(1)
    pt.backward(torch.tensor(dp))
    assert np.allclose(p, pt.detach().numpy())
    assert np.allclose(L.avgpool_backward(dp, c), at.grad.permute(0, 2, 3, 1).numpy())


# ------------------------------------------------------------------ GELU, residual linear
def test_gelu_closed_forms_and_library():
    z = np.linspace(-6, 6, 97)
    g = L.gelu(z)
    assert L.gelu(np.zeros(1))[0] == 0.0
    assert np.allclose(g - L.gelu(-z), z, atol=1e-15)             # z Phi(z) - (-z) Phi(-z) = z
    assert abs(L.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    zt = torch.tensor(z, requires_grad=True)
    yt = F.gelu(zt)
    yt.sum().backward()
    assert _rel(g, yt.detach().numpy()) < 1e-14
    assert _rel(L.gelu_derivative(z), zt.grad.numpy()) < 1e-13


def test_linear_gelu_rows_and_residual_against_library_and_fd():
    rng = np.random.default_rng(20)
    B, rows, din, dout = 2, 3, 5, 5
    x = rng.standard_normal((B, rows * din)); w = rng.standard_normal((dout, din)); b = rng.standard_normal(dout)
    skip = rng.standard_normal((B, rows * dout)); r = rng.standard_normal((B, rows * dout))
    y, c = L.linear_forward(x, w, b, False, "gelu", rows, None)
    dx, dw, db = L.linear_backward(r, c, w, False, "gelu")
    xt, wt, bt = (torch.tensor(a, requires_grad=True) for a in (x, w, b))
    yt = F.gelu(F.linear(xt.reshape(B * rows, din), wt, bt)).reshape(B, -1)
    yt.backward(torch.tensor(r))
    assert _rel(y, yt.detach().numpy()) < 1e-13
    assert _rel(dx, xt.grad.numpy()) < 1e-12 and _rel(dw, wt.grad.numpy()) < 1e-12 and _rel(db, bt.grad.numpy()) < 1e-12
    f = lambda: float((L.linear_forward(x, w, b, False, "gelu", rows, None)[0] * r).sum())
    assert _rel(dx, _fd(f, x)) < 1e-6
    # residual: the result is the plain layer plus the skipped tensor
    y2, _ = L.linear_forward(x, w, b, False, None, rows, skip)
    y1, _ = L.linear_forward(x, w, b, False, None, rows, None)
    assert np.allclose(y2, y1 + skip)


# ------------------------------------------------------------------ layer normalisation
def test_layernorm_invariants_library_and_fd():
    rng = np.random.default_rng(21)
    B, rows, d = 2, 3, 7
    x = rng.standard_normal((B, rows * d)) * 3 + 1
    gam = rng.standard_normal(d); bet = rng.standard_normal(d); r = rng.standard_normal((B, rows * d))
    y1, c1 = L.layernorm_forward(x, np.ones(d), np.zeros(d), d, eps=0.0)
    y1 = y1.reshape(-1, d)
    assert np.allclose(y1.mean(axis=1), 0, atol=1e-14) and np.allclose((y1 ** 2).mean(axis=1), 1, atol=1e-12)
    y, c = L.layernorm_forward(x, gam, bet, d, 1e-5)
    dx, dg, db = L.layernorm_backward(r, c, gam)
    xt, gt, bt = (torch.tensor(a, requires_grad=True) for a in (x, gam, bet))
    yt = F.layer_norm(xt.reshape(-1, d), (d,), gt, bt, 1e-5).reshape(B, -1)
    yt.backward(torch.tensor(r))
    assert _rel(y, yt.detach().numpy()) < 1e-13
    assert _rel(dx, xt.grad.numpy()) < 1e-11 and _rel(dg, gt.grad.numpy()) < 1e-12 and _rel(db, bt.grad.numpy()) < 1e-12
    f = lambda: float((L.layernorm_forward(x, gam, bet, d, 1e-5)[0] * r).sum())
    assert _rel(dx, _fd(f, x)) < 1e-6
    assert _rel(dg, _fd(f, gam)) < 1e-7
    # dx comes from the gain passed to backward, the statistics from the forward pass
    gam2 = rng.standard_normal(d)
    dx2, _, _ = L.layernorm_backward(r, c, gam2)
    dxr, _, _ = L.layernorm_backward((r.reshape(-1, d) * gam2 / gam).reshape(r.shape), c, gam)
    assert np.allclose(dx2, dxr)


# ------------------------------------------------------------------ attention
def _attention_loops(qkv, s, d, heads):
    """Definition written out with loops (tiny sizes only)."""
    B = qkv.shape[0]
    dh = d // heads
    t = qkv.reshape(B, s, 3, heads, dh)
    out = np.zeros((B, s, heads, dh))
    for b in range(B):
        for h in range(heads):
            for i in range(s):
                sc = np.array([t[b, i, 0, h] @ t[b, j, 1, h] / np.sqrt(dh) for j in range(i + 1)])
                p = np.exp(sc - sc.max())
                p /= p.sum()
                for j in range(i + 1):
                    out[b, i, h] += p[j] * t[b, j, 2, h]
    return out.reshape(B, s * d)


def test_attention_definition_causality_library_and_fd():
    rng = np.random.default_rng(22)
    B, s, d, heads = 2, 5, 6, 2
    qkv = rng.standard_normal((B, s * 3 * d)); r = rng.standard_normal((B, s * d))
    y, c = L.attention_forward(qkv, s, d, heads)
    assert np.allclose(y, _attention_loops(qkv, s, d, heads), atol=1e-13)
    assert np.allclose(c["p"].sum(axis=-1), 1.0) and np.all(np.triu(c["p"], 1) == 0.0)
    # position i depends on positions <= i only
    q2 = qkv.reshape(B, s, 3 * d).copy()
    q2[:, 3:] += rng.standard_normal((B, s - 3, 3 * d))
    y2, _ = L.attention_forward(q2.reshape(B, -1), s, d, heads)
    assert np.allclose(y.reshape(B, s, d)[:, :3], y2.reshape(B, s, d)[:, :3])
    # first position attends to itself only: output = its own value vector
    assert np.allclose(y.reshape(B, s, d)[:, 0], qkv.reshape(B, s, 3, d)[:, 0, 2])
    dx = L.attention_backward(r, c)
    dh = d // heads
    tt = torch.tensor(qkv.reshape(B, s, 3, heads, dh), requires_grad=True)
    qh, kh, vh = (tt[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    yt = F.scaled_dot_product_attention(qh, kh, vh, is_causal=True).permute(0, 2, 1, 3).reshape(B, s * d)
    yt.backward(torch.tensor(r))
    assert _rel(y, yt.detach().numpy()) < 1e-12
    assert _rel(dx, tt.grad.numpy().reshape(B, -1)) < 1e-11
    f = lambda: float((L.attention_forward(qkv, s, d, heads)[0] * r).sum())
    assert _rel(dx, _fd(f, qkv)) < 1e-6


# ------------------------------------------------------------------ embedding
def test_embedding_definition_and_gradients():
    rng = np.random.default_rng(23)
    B, s, d, vocab = 3, 4, 5, 6
    tok = rng.integers(0, vocab, (B, s)); tok[0, 0] = tok[1, 2] = tok[2, 3] = 1     # repeated token
    wte = rng.standard_normal((vocab, d)); wpe = rng.standard_normal((s, d)); r = rng.standard_normal((B, s * d))
    y, c = L.embedding_forward(tok, wte, wpe)
    for b in range(B):
        for i in range(s):
            assert np.array_equal(y.reshape(B, s, d)[b, i], wte[tok[b, i]] + wpe[i])
    dwte, dwpe = L.embedding_backward(r, c, vocab, d)
    f = lambda: float((L.embedding_forward(tok, wte, wpe)[0] * r).sum())
    assert _rel(dwte, _fd(f, wte)) < 1e-8 and _rel(dwpe, _fd(f, wpe)) < 1e-8
    assert np.allclose(dwte[1], sum(r.reshape(B, s, d)[b, i] for b in range(B) for i in range(s) if tok[b, i] == 1))
