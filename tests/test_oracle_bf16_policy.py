"""Pins of WHERE the oracle rounds to bfloat16 under precision="bf16" (the mixed-precision contract: bf16
activations and propagated gradients, fp32 master weights, momentum and weight gradients, sums in high precision).

The contract, stated once more here and evaluated independently of oracle/stage.py and oracle/layers.py with CPU
library tensors (fp64 arithmetic, library layer functions, library derivatives through autograd of ONE layer at a
time, `.to(bfloat16)` exactly at the stored tensors and nowhere else):

  stored, hence on the bf16 grid:
    * the stage input (except integer tokens);
    * the working copy of every contraction operand: dense weights, filters, both embedding tables;
    * every layer's result -- except the logits, which feed the loss directly and stay unrounded;
    * the pre-activation a GELU layer keeps for its derivative;
    * every propagated gradient: the gradient of a layer result (and of the stage input).  A result read by several
      layers collects their contributions in reverse layer order, and the stored sum is rounded after each one;
  NOT rounded: biases, gains and shifts of normalisation / affine layers (read from the fp32 masters), the
  statistics of layer normalisation, softmax probabilities, weight gradients, momentum, master weights.
  Decisions (ReLU masks, pooling winners) are taken on the stored values.

Comparisons are to 1e-9: the two sides make the same roundings, so they differ by fp64 rounding only, while a
rounding dropped or added anywhere moves values by 2^-9 relative.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle.precision import round_to_bf16
from oracle.stage import Stage as OStage
from workloads.configs import (affine, attention, avgpool, bottleneck, conv, embedding, layernorm, linear, maxpool,
                               softmax_ce, transformer_block)
from workloads.synth import param_shapes

EXACT = 1e-9


def stored(t):
    return t.to(torch.bfloat16).to(torch.float64)


def T(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float64)))


def on_grid(a):
    a = np.asarray(a, dtype=np.float64)
    return np.array_equal(round_to_bf16(a), a)


# ---------------------------------------------------------------- the contract, second statement
def layer_function(sp, p):
    """The layer as a function of its input tensors (library ops, fp64); operands the contract stores are rounded
    by the caller.  Returns f(inputs...) -> unrounded result."""
    k = sp["kind"]
    if k == "linear":
        w, b = stored(T(p["w"])), T(p["b"])
        rows = sp.get("rows", 1)

        def f(x, skip=None, z_override=None):
            z = F.linear(x.reshape(x.shape[0] * rows, -1), w, b)
            if sp["relu"]:
                y = torch.relu(z)
            elif sp.get("act") == "gelu":
                y = F.gelu(z)
            else:
                y = z
            if skip is not None:
                y = y + skip.reshape(y.shape)
            return y.reshape(x.shape[0], -1)
        return f
    if k == "conv":
        w, b = stored(T(p["w"])).permute(0, 3, 1, 2), T(p["b"])

        def f(x):
            x4 = x.reshape(x.shape[0], sp["h"], sp["w"], sp["cin"]).permute(0, 3, 1, 2)
            y = F.conv2d(x4, w, b, stride=sp["stride"], padding=sp["pad"]).permute(0, 2, 3, 1)
            return (torch.relu(y) if sp["relu"] else y).reshape(x.shape[0], -1)
        return f
    if k == "maxpool":
        def f(x):
            x4 = x.reshape(x.shape[0], sp["h"], sp["w"], sp["c"]).permute(0, 3, 1, 2)
            return F.max_pool2d(x4, sp["k"], sp["stride"], sp.get("pad", 0)).permute(0, 2, 3, 1).reshape(x.shape[0], -1)
        return f
    if k == "affine":
        g, s = T(p["w"]), T(p["b"])

        def f(x):
            y = x.reshape(-1, sp["c"]) * g + s
            return (torch.relu(y) if sp["relu"] else y).reshape(x.shape[0], -1)
        return f
    if k == "resadd":
        def f(a, b):
            y = a + b.reshape(a.shape)
            return torch.relu(y) if sp["relu"] else y
        return f
    if k == "avgpool":
        return lambda x: x.reshape(x.shape[0], sp["h"] * sp["w"], sp["c"]).mean(dim=1)
    if k == "layernorm":
        g, s = T(p["w"]), T(p["b"])
        return lambda x: F.layer_norm(x.reshape(-1, sp["d"]), (sp["d"],), g, s, sp["eps"]).reshape(x.shape)
    if k == "attention":
        s_, d, h = sp["s"], sp["d"], sp["heads"]
        dh = d // h

        def f(x):
            t = x.reshape(x.shape[0], s_, 3, h, dh)
            q, kk, v = (t[:, :, i].transpose(1, 2) for i in range(3))
            sc = q @ kk.transpose(-1, -2) / np.sqrt(dh)
            sc = sc.masked_fill(torch.triu(torch.ones(s_, s_, dtype=torch.bool), 1), float("-inf"))
            return (torch.softmax(sc, dim=-1) @ v).transpose(1, 2).reshape(x.shape[0], s_ * d)
        return f
    raise ValueError(k)


class PolicyReference:
    """One stage under the contract above.  forward() keeps, per layer, the stored input tensors; backward() takes
    one layer at a time: library derivative of that layer at its stored inputs, then the storage rule for gradients."""

    def __init__(self, specs, params, M, N):
        self.specs, self.params, self.M, self.N = specs, params, M, N
        self.saved = {}

    def sources(self, li):
        """Indices of the results layer li reads (-1: the stage input), first operand first."""
        sp = self.specs[li]
        if sp["kind"] == "conv" and sp.get("src", 1) != 1:
            return [li - sp["src"]]
        if sp["kind"] == "resadd":
            return [li - 1, li - sp["src_b"]]
        if sp["kind"] == "linear" and sp.get("skip"):
            return [li - 1, li - sp["skip"] - 1]     # the input of the layer `skip` positions before
        return [li - 1]

    def forward_micro(self, slot, x, labels=None):
        specs = self.specs
        res = {-1: T(x).long() if specs[0]["kind"] == "embedding" else stored(T(x)).reshape(len(x), -1)}
        zs = {}
        for li, (sp, p) in enumerate(zip(specs, self.params)):
            k = sp["kind"]
            ins = [res[max(t, -1)] for t in self.sources(li)]
            if k == "embedding":
                out = F.embedding(ins[0], stored(T(p["w"]))) + stored(T(p["b"]))[None, :sp["s"], :]
                out = out.reshape(out.shape[0], -1)
            elif k == "softmax_ce":
                rows = sp.get("rows", 1)
                lab = torch.from_numpy(np.asarray(labels).reshape(-1).astype(np.int64))
                loss = F.cross_entropy(ins[0].reshape(len(lab), -1), lab, reduction="mean")
                self.saved[slot] = (res, zs, lab)
                return ins[0].numpy(), float(loss)
            else:
                out = layer_function(sp, p)(*ins)
                if k == "linear" and sp.get("act") == "gelu":
                    zs[li] = stored(F.linear(ins[0].reshape(-1, sp["din"]), stored(T(p["w"])), T(p["b"])))
            feeds_loss = li + 1 < len(specs) and specs[li + 1]["kind"] == "softmax_ce"
            res[li] = out if feeds_loss else stored(out)
        self.saved[slot] = (res, zs, None)
        return res[len(specs) - 1].numpy()

    def backward(self, slots, dy=None):
        specs = self.specs
        n_l = len(specs)
        micro = self.M // self.N
        wsum = [None] * n_l
        dxs = []
        for i, slot in enumerate(slots):
            res, zs, lab = self.saved.pop(slot)
            grad = {}

            def give(t, c):
                t = max(t, -1)
                c = c.reshape(c.shape[0], -1)
                grad[t] = stored(c) if t not in grad else stored(grad[t] + c)

            if dy is not None:
                give(n_l - 1, T(dy[i * micro:(i + 1) * micro]))
            # contributions must reach a shared result in reverse order of its READERS; a linear layer with a skip
            # connection is a reader of its skip source, and hands it the incoming gradient as it is
            for li in range(n_l - 1, -1, -1):
                sp, p = specs[li], self.params[li]
                k = sp["kind"]
                src = self.sources(li)
                if k == "softmax_ce":
                    logits = res[li - 1].detach().clone().requires_grad_(True)
                    rows = sp.get("rows", 1)
                    loss = F.cross_entropy(logits.reshape(len(lab), -1), lab, reduction="sum") / (self.M * rows)
                    give(li - 1, torch.autograd.grad(loss, logits)[0])
                    continue
                g = grad.pop(li)
                if k == "embedding":
                    wte = stored(T(p["w"])).requires_grad_(True)
                    wpe = stored(T(p["b"])).requires_grad_(True)
                    out = (F.embedding(res[-1], wte) + wpe[None, :sp["s"], :]).reshape(g.shape)
                    gw, gb = torch.autograd.grad(out, [wte, wpe], grad_outputs=g)
                    self._acc(wsum, li, gw, gb)
                    continue
                ins = [res[max(t, -1)].detach().clone().requires_grad_(True) for t in src]
                leaves = list(ins)
                pw = None
                if p:
                    # the derivative w.r.t. the weights is taken at the operand the layer read (the stored copy)
                    roundw = k in ("linear", "conv")
                    pw = [(stored(T(p["w"])) if roundw else T(p["w"])).requires_grad_(True), T(p["b"]).requires_grad_(True)]
                    leaves += pw
                out = self._apply(sp, pw, ins, zs.get(li))
                gs = torch.autograd.grad(out, leaves, grad_outputs=g.reshape(out.shape), allow_unused=True)
                if k == "linear" and sp.get("skip"):
                    give(src[1], gs[1])          # reader with the higher index: first
                    give(src[0], gs[0])
                elif k == "resadd":
                    give(src[1], gs[1])
                    give(src[0], gs[0])
                else:
                    give(src[0], gs[0])
                if p:
                    self._acc(wsum, li, gs[-2], gs[-1])
            dxs.append(grad.get(-1))
        self.grads = wsum
        return None if dxs[0] is None else torch.cat(dxs).numpy()

    @staticmethod
    def _acc(wsum, li, gw, gb):
        if wsum[li] is None:
            wsum[li] = {"w": gw.numpy().copy(), "b": gb.numpy().copy()}
        else:
            wsum[li]["w"] += gw.numpy()
            wsum[li]["b"] += gb.numpy()

    @staticmethod
    def _apply(sp, pw, ins, z_stored):
        """The layer as a differentiable function of (inputs, parameters given as leaves)."""
        k = sp["kind"]
        x = ins[0]
        if k == "linear":
            rows = sp.get("rows", 1)
            z = F.linear(x.reshape(x.shape[0] * rows, -1), pw[0], pw[1])
            if sp["relu"]:
                y = torch.relu(z)
            elif sp.get("act") == "gelu":
                # the derivative of the activation is evaluated at the STORED pre-activation
                zs_ = z_stored.detach().clone().requires_grad_(True)
                dact = torch.autograd.grad(F.gelu(zs_).sum(), zs_)[0]
                y = z * dact.detach()       # same derivative w.r.t. z as gelu at the stored point
            else:
                y = z
            if len(ins) > 1:
                y = y + ins[1].reshape(y.shape)
            return y.reshape(x.shape[0], -1)
        if k == "conv":
            x4 = x.reshape(x.shape[0], sp["h"], sp["w"], sp["cin"]).permute(0, 3, 1, 2)
            y = F.conv2d(x4, pw[0].permute(0, 3, 1, 2), pw[1], stride=sp["stride"], padding=sp["pad"]).permute(0, 2, 3, 1)
            return (torch.relu(y) if sp["relu"] else y).reshape(x.shape[0], -1)
        if k == "affine":
            y = x.reshape(-1, sp["c"]) * pw[0] + pw[1]
            return (torch.relu(y) if sp["relu"] else y).reshape(x.shape[0], -1)
        if k == "layernorm":
            return F.layer_norm(x.reshape(-1, sp["d"]), (sp["d"],), pw[0], pw[1], sp["eps"]).reshape(x.shape)
        return layer_function(sp, None)(*ins)


# ---------------------------------------------------------------- networks and inputs (deliberately OFF the grid)
def rand_params(specs, rng):
    ps = []
    for sp in specs:
        shp = param_shapes(sp)
        p = {}
        if shp and sp["kind"] in ("layernorm", "affine"):
            p["w"] = 1.0 + 0.3 * rng.standard_normal(shp["w"])
            p["b"] = 0.2 * rng.standard_normal(shp["b"])
        elif shp and sp["kind"] == "embedding":
            p["w"], p["b"] = 0.7 * rng.standard_normal(shp["w"]), 0.7 * rng.standard_normal(shp["b"])
        elif shp:
            p["w"] = rng.standard_normal(shp["w"]) * np.sqrt(2.0 / np.prod(shp["w"][1:]))
            p["b"] = 0.3 * rng.standard_normal(shp["b"])
        ps.append({k: v.astype(np.float32).astype(np.float64) for k, v in p.items()})   # fp32 masters
    return ps


def transformer_stage(last):
    s, d, heads, ffn, vocab = 6, 16, 2, 24, 11
    specs = [embedding(vocab, s, d)] + transformer_block(s, d, heads, ffn) + transformer_block(s, d, heads, ffn)
    if last:
        specs += [layernorm(d, s), linear(d, vocab, False, rows=s), softmax_ce(vocab, rows=s)]
    return specs, vocab, s


def residual_stage(last):
    specs = [conv(9, 9, 3, 8, 3, 1, 1, True), maxpool(9, 9, 8, 3, 2, 1)]
    b1, h, c = bottleneck(5, 8, 4, 2, True)
    b2, h, c = bottleneck(h, c, 4, 1, False)
    specs += b1 + b2
    if last:
        specs += [avgpool(h, h, c), linear(c, 7, True), linear(7, 5, False), softmax_ce(5)]
    return specs, h * h * c


def run_both(specs, x, labels, dy, M, N, seed):
    rng = np.random.default_rng(seed)
    ps = rand_params(specs, rng)
    o = OStage(specs, ps, 0.05, 0.9, M, N, precision="bf16")
    r = PolicyReference(specs, ps, M, N)
    micro = M // N
    last = specs[-1]["kind"] == "softmax_ce"
    for j in range(N):
        rows = slice(j * micro, (j + 1) * micro)
        if last:
            oy, ol = o.forward_micro(j, x[rows], labels[rows])
            ry, rl = r.forward_micro(j, x[rows], labels[rows])
            assert abs(ol - rl) <= EXACT * abs(rl)
            assert not on_grid(oy), "the logits feed the loss directly and are not rounded"
        else:
            oy, ry = o.forward_micro(j, x[rows]), r.forward_micro(j, x[rows])
            assert on_grid(oy), "a stage output is a stored tensor"
        np.testing.assert_allclose(oy.reshape(ry.shape), ry, rtol=EXACT, atol=1e-300)
    return o, r


def check_backward(o, r, N, dy):
    odx, rdx = o.backward(list(range(N)), dy), r.backward(list(range(N)), dy)
    if rdx is None:
        assert odx is None
    else:
        assert on_grid(odx), "the gradient handed to the worker before is a stored tensor"
        np.testing.assert_allclose(odx.reshape(rdx.shape), rdx, rtol=EXACT, atol=1e-300)
    for li, (og, rg) in enumerate(zip(o.grads, r.grads)):
        assert (og is None) == (rg is None), li
        if og is None:
            continue
        for k in og:
            scale = np.max(np.abs(rg[k])) + 1e-300
            assert np.max(np.abs(og[k].reshape(rg[k].shape) - rg[k])) <= EXACT * scale, (li, k)
            assert not on_grid(og[k]), "weight gradients are not rounded"


@pytest.mark.parametrize("last", [True, False])
def test_transformer_stage_rounds_where_the_contract_says(last):
    specs, vocab, s = transformer_stage(last)
    M, N = 4, 2
    rng = np.random.default_rng(1)
    x = rng.integers(0, vocab, (M, s)).astype(np.int32)
    labels = rng.integers(0, vocab, (M, s)).astype(np.int32)
    dy = None if last else rng.standard_normal((M, s * 16)) / M      # off the grid: rounded when it is taken in
    o, r = run_both(specs, x, labels, dy, M, N, 2)
    # what the backward pass keeps: layer results on the grid, statistics and probabilities not
    caches = o.stash[0]
    for li, sp in enumerate(specs):
        c = caches[li]
        if sp["kind"] == "layernorm":
            assert not on_grid(c["rstd"]) and not on_grid(c["xhat"])
        if sp["kind"] == "attention":
            assert not on_grid(c["p"]) and on_grid(c["q"]) and on_grid(c["v"])
        if sp["kind"] == "linear" and sp.get("act") == "gelu":
            assert on_grid(c["z"])
        if sp["kind"] == "linear":
            assert on_grid(c["x"])
    check_backward(o, r, N, dy)


@pytest.mark.parametrize("last", [True, False])
def test_residual_stage_rounds_where_the_contract_says(last):
    specs, out_elems = residual_stage(last)
    M, N = 4, 2
    rng = np.random.default_rng(3)
    x = rng.standard_normal((M, 9, 9, 3))                             # off the grid: rounded when it is taken in
    labels = rng.integers(0, 5, M).astype(np.int32)
    dy = None if last else rng.standard_normal((M, out_elems)) / M
    o, r = run_both(specs, x, labels, dy, M, N, 4)
    caches = o.stash[0]
    for li, sp in enumerate(specs):
        if sp["kind"] in ("conv", "affine", "resadd"):
            assert on_grid(caches[li]["y"]), (li, sp["kind"])
    check_backward(o, r, N, dy)


def test_update_keeps_masters_and_momentum_unrounded():
    specs = [linear(5, 4, True), linear(4, 3, False), softmax_ce(3)]
    rng = np.random.default_rng(5)
    ps = rand_params(specs, rng)
    o = OStage(specs, ps, 0.05, 0.9, 4, 2, precision="bf16")
    x, lab = rng.standard_normal((4, 5)), rng.integers(0, 3, 4)
    for j in range(2):
        o.forward_micro(j, x[2 * j:2 * j + 2], lab[2 * j:2 * j + 2])
    o.backward([0, 1])
    g = [{k: v.copy() for k, v in gr.items()} for gr in o.grads[:2]]
    o.update()
    for li in range(2):
        for k in ("w", "b"):
            assert np.array_equal(o.bufs[li][k], g[li][k])                       # buf_1 = g, unrounded
            assert np.array_equal(o.params[li][k], ps[li][k] - 0.05 * g[li][k])  # the master moves by the exact step
            assert not on_grid(o.params[li][k])


def test_two_layer_case_by_hand():
    """One sample, 2 -> 1 -> 1, ReLU in between, numbers chosen so that every rounding changes a value.
    bf16 keeps 8 significant bits: spacing 2^-7 in [1, 2), 2^-8 in [0.5, 1), 2^-6 in [2, 4)."""
    x = np.array([[1.00390625, 3.0]])                  # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: to even, 1.0
    w1 = np.array([[1.0078125 + 2.0 ** -9, 0.5]])      # 1 + 2^-7 + 2^-9 -> 1.0078125 (below the tie)
    b1 = np.array([0.001])                             # not rounded
    w2 = np.array([[0.75]])
    b2 = np.array([0.0])
    specs = [linear(2, 1, True), linear(1, 1, False)]
    o = OStage(specs, [{"w": w1, "b": b1}, {"w": w2, "b": b2}], 0.1, 0.0, 1, 1, precision="bf16")
    y = o.forward_micro(0, x)
    # layer 1: 1.0 * 1.0078125 + 3 * 0.5 + 0.001 = 2.5088125 -> spacing 2^-6 = 0.015625: 2.5 + 0.0088 -> 2.515625
    h = 2.515625
    assert o.stash[0][0]["y"][0, 0] == h
    # layer 2: 0.75 * 2.515625 = 1.88671875 -> spacing 2^-7: 1.8828125 + 0.0039 = 1.8867 is the tie of 1.8828125 and
    # 1.890625 (1.88671875 exactly): to even.  1.8828125 = 241 * 2^-7 (odd), 1.890625 = 242 * 2^-7 (even)
    assert y[0, 0] == 1.890625
    dy = np.array([[0.3]])                             # -> 0.30078125 (spacing 2^-9 in [0.25, 0.5): 154 * 2^-9)
    dx = o.backward([0], dy)
    g = 0.30078125
    # layer 2: dW2 = g * h (unrounded), gradient to h = g * 0.75 = 0.2255859375 -> spacing 2^-10: 231 * 2^-10 exactly
    assert o.grads[1]["w"][0, 0] == g * h and o.grads[1]["b"][0] == g
    gh = 0.2255859375
    # layer 1: dW1 = gh * x_stored (unrounded), dx = gh * w1_stored -> rounded
    assert np.array_equal(o.grads[0]["w"], np.array([[gh * 1.0, gh * 3.0]]))
    want = round_to_bf16(np.array([[gh * 1.0078125, gh * 0.5]]))
    assert np.array_equal(dx, want) and dx[0, 0] == 0.2275390625    # 0.22734... -> 233 * 2^-10
