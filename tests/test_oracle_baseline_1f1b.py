"""Pins of the oracle's PipeDream-style baseline (oracle/baseline.py): the 1F1B schedule against what the paper and
the cited system state about it, and the training rule against an independent evaluation.

  * schedule: worker s (from 0) makes W - s forward passes before its first backward pass and then takes them in turn;
    the last worker alternates from the start; in the steady state a batch leaves every 2 time-points; a backward pass
    reads the version its forward pass read (horizontal weight stashing), which is max(0, b - (W - s)) updates for
    batch b on worker s; W - s - 1 older versions are kept and W - s batches are in flight on worker s;
  * the paper's figure of PipeDream with four workers: batch 3 makes its backward pass on the version its forward
    pass used although the update of batch 2 is already there;
  * K = 1 is plain sequential SGD with momentum (library autograd and a hand-written momentum step);
  * K = 3: because a batch is differentiated at the very weights its forward pass used, its gradient is the exact
    gradient of the loss of the WHOLE network at the composite weights (W_0(v_0), W_1(v_1), W_2(v_2)) with
    v_s = max(0, b - 1 - (W - s - 1)): evaluated with library autograd on the network in one piece and applied in
    batch order, this reproduces every weight of the oracle's run (the update rule of PipeDream).
"""
import numpy as np
import pytest
import torch

from oracle import baseline as BL
from oracle.schedule import BWD, FWD
from workloads.configs import linear, softmax_ce


@pytest.mark.parametrize("W", [1, 2, 3, 4, 6])
def test_schedule_is_1f1b_with_horizontal_stashing(W):
    n = 3 * W + 5
    ops = BL.simulate_1f1b(W, n)
    per = {s: [(t, kind, b, read, live) for (t, w, kind, b, _, read, live) in ops if w == s] for s in range(W)}
    for s in range(W):
        kinds = [k for (_, k, _, _, _) in per[s]]
        first_b = kinds.index(BWD)
        assert first_b == W - s and all(k == FWD for k in kinds[:first_b])           # start-up depth
        body = kinds[first_b:len(kinds) - (W - s - 1)] if W - s - 1 else kinds[first_b:]
        assert all(body[i] != body[i + 1] for i in range(len(body) - 1))             # then one backward, one forward in turn
        fw = {b: (t, read) for (t, k, b, read, _) in per[s] if k == FWD}
        for (t, k, b, read, live) in per[s]:
            if k == FWD:
                assert read == live == max(0, b - (W - s))
            else:
                assert read == fw[b][1] and t > fw[b][0]                               # the version of its forward pass
                assert live == b - 1                                                   # updates land in batch order
        assert [b for (_, k, b, _, _) in per[s] if k == FWD] == list(range(1, n + 1))
        assert [b for (_, k, b, _, _) in per[s] if k == BWD] == list(range(1, n + 1))
    # a forward pass reaches worker s+1 one time-point after worker s at the earliest, a backward pass worker s-1 likewise
    when = {(w, kind, b): t for (t, w, kind, b, _, _, _) in ops}
    for b in range(1, n + 1):
        for s in range(W - 1):
            assert when[(s + 1, FWD, b)] > when[(s, FWD, b)] and when[(s, BWD, b)] > when[(s + 1, BWD, b)]
        assert when[(W - 1, BWD, b)] == when[(W - 1, FWD, b)] + 1                      # backward right after forward
    done = [when[(0, BWD, b)] for b in range(1, n + 1)]
    assert all(b - a == 2 for a, b in zip(done[W:-W], done[W + 1:-W])) or n < 3 * W    # one batch per two time-points
    assert BL.versions_kept(W, n) == [W - s - 1 for s in range(W)]
    assert BL.batches_in_flight(W, n) == [W - s for s in range(W)]


def test_the_papers_pipedream_figure():
    # four workers: when batch 3 makes its backward pass on the first worker, the update of batch 2 has been applied
    # there, yet the pass reads the weights of its forward pass, which no update had reached
    ops = BL.simulate_1f1b(4, 8)
    b3 = [o for o in ops if o[1] == 0 and o[2] == BWD and o[3] == 3][0]
    assert b3[6] == 2 and b3[5] == 0
    f5 = [o for o in ops if o[1] == 0 and o[2] == FWD and o[3] == 5][0]
    assert f5[5] == 1       # the fifth batch is the first to see an update on the first worker


def _mlp_stages(K):
    layers = [linear(12, 16, True), linear(16, 16, True), linear(16, 16, True), linear(16, 5, False), softmax_ce(5)]
    cuts = {1: [layers], 2: [layers[:2], layers[2:]], 3: [layers[:1], layers[1:3], layers[3:]]}[K]
    rng = np.random.default_rng(K)
    params = [[({"w": rng.standard_normal((sp["dout"], sp["din"])) * np.sqrt(2.0 / sp["din"]), "b": 0.1 * rng.standard_normal(sp["dout"])}
                if sp["kind"] == "linear" else {}) for sp in st] for st in cuts]
    batches = [(rng.standard_normal((6, 12)), rng.integers(0, 5, 6)) for _ in range(9)]
    return cuts, params, batches


def _whole_network_loss(ws, x, y):
    a = torch.from_numpy(x)
    for i, (w, b) in enumerate(ws):
        a = torch.nn.functional.linear(a, w, b)
        if i < len(ws) - 1:
            a = torch.relu(a)
    return torch.nn.functional.cross_entropy(a, torch.from_numpy(y).long())


@pytest.mark.parametrize("K", [1, 2, 3])
def test_training_rule_against_whole_network_autograd_at_the_stashed_weights(K):
    cuts, params, batches = _mlp_stages(K)
    lr, mu = 0.05, 0.9
    got = BL.run_1f1b(cuts, params, batches, lr, mu)
    # independent evaluation: versions[s][v] = parameters of worker s after v updates
    versions = [[[(torch.tensor(p["w"]), torch.tensor(p["b"])) for p in st if p]] for st in params]
    bufs = [[(torch.zeros_like(w), torch.zeros_like(b)) for (w, b) in v[0]] for v in versions]
    losses = []
    for bi, (x, y) in enumerate(batches, start=1):
        read = [max(0, bi - (K - s)) for s in range(K)]
        leaves = [[(w.clone().requires_grad_(True), b.clone().requires_grad_(True)) for (w, b) in versions[s][read[s]]] for s in range(K)]
        loss = _whole_network_loss([wb for st in leaves for wb in st], x, y)
        losses.append(float(loss.detach()))
        loss.backward()
        for s in range(K):
            live = versions[s][bi - 1]          # every worker has applied the updates of the batches before this one
            new = []
            for li, ((w, b), (gw, gb)) in enumerate(zip(live, leaves[s])):
                mw, mb = bufs[s][li]
                mw, mb = mu * mw + gw.grad, mu * mb + gb.grad
                bufs[s][li] = (mw, mb)
                new.append((w - lr * mw, b - lr * mb))
            versions[s].append(new)
    np.testing.assert_allclose(got["losses"], losses, rtol=1e-10)
    for s in range(K):
        want = versions[s][len(batches)]
        have = [p for p in got["stages"][s].params if p]
        for (w, b), p in zip(want, have):
            np.testing.assert_allclose(p["w"], w.numpy(), rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(p["b"], b.numpy(), rtol=1e-9, atol=1e-12)
    if K == 1:
        # one worker: nothing is stale, every backward pass reads the live weights
        assert all(read == live for (_, _, _, _, _, read, live) in got["ops"])


def test_stale_backward_differs_from_the_live_one():
    # the same run with backward passes on the LIVE weights (what TiMePReSt does) gives other weights: the stashing is real
    cuts, params, batches = _mlp_stages(3)
    a = BL.run_1f1b(cuts, params, batches, 0.05, 0.9)
    ops = BL.simulate_1f1b(3, len(batches))
    assert any(read != live for (_, _, kind, _, _, read, live) in ops if kind == BWD)
    from oracle.stage import Stage
    stages = [Stage(cuts[s], params[s], 0.05, 0.9, 6, 1, "f64") for s in range(3)]
    fo, bo = {}, {}
    for (t, s, kind, b, _, read, live) in ops:
        x, y = batches[b - 1]
        if kind == FWD:
            xin = x if s == 0 else fo.pop((b, s - 1))
            out = stages[s].forward_micro(b, xin, y) if s == 2 else stages[s].forward_micro(b, xin)
            if s < 2:
                fo[(b, s)] = out
        else:
            dx = stages[s].backward([b], None if s == 2 else bo.pop((b, s + 1)))
            if s > 0:
                bo[(b, s)] = dx
            stages[s].update()
    assert np.max(np.abs(stages[0].params[0]["w"] - a["stages"][0].params[0]["w"])) > 1e-6
