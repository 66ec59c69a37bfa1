"""Training with different version differences v (the comparative study the paper leaves as future work, section
"Version Difference"): the same 7-layer network and data, cut into W = 1, 3, 4 and 7 stages with N = 2 micro-batches,
which gives v = 1, 1, 2 and 3.  Pins that hold whatever v is:

* the first mini-batch sees the initial weights on every worker, so its loss does not depend on W;
* W = 1 is plain sequential SGD with momentum;
* with N = 2 a forward pass of mini-batch b on worker s reads weights that lack the updates of the W - 1 - s
  mini-batches in flight below it, while every backward pass reads all b - 1 earlier updates (zero staleness);
* training still converges for v = 2 and 3 at a small learning rate; the deepest pipeline drifts furthest from the
  sequential trajectory (lr 0.005: mean |loss - sequential loss| 0.074, 0.075, 0.146 for v = 1, 2, 3; at lr 0.02 the
  runs with stale forward passes stall, which is the cost the paper's follow-up study would quantify).
"""
import numpy as np
import pytest

from oracle import pipeline
from oracle import schedule as S
from workloads import Config, init_params, make_batch
from workloads.configs import linear, softmax_ce

LAYERS = [linear(32, 32, True) for _ in range(6)] + [linear(32, 10, False), softmax_ce(10)]


def cut(W):
    """W stages of consecutive layers; the loss layer stays with the last linear layer."""
    body = LAYERS[:-1]
    per, extra = divmod(len(body), W)
    stages, at = [], 0
    for s in range(W):
        n = per + (1 if s < extra else 0)
        stages.append(body[at:at + n])
        at += n
    stages[-1] = stages[-1] + [LAYERS[-1]]
    return stages


def train(W, steps=80, N=2, vertical_sync=False):
    cfg = Config(name="study", dtype="f32", M=8, N=N, stages=cut(W), in_shape=(32,), classes=10, seed=11, lr=0.005)
    params = init_params(cfg, bias_std=0.05)
    batches = [make_batch(cfg, i % 8) for i in range(steps)]   # 8 distinct mini-batches, revisited
    return cfg, pipeline.run(cfg, params, batches, vertical_sync=vertical_sync)


RUNS = {}


def run_of(W):
    if W not in RUNS:
        RUNS[W] = train(W)
    return RUNS[W]


@pytest.mark.parametrize("W,v", [(3, 1), (4, 2), (7, 3)])
def test_version_difference_of_the_cuts(W, v):
    assert S.version_difference_simulated(W, 2) == v


def test_first_loss_does_not_depend_on_the_cut():
    first = [run_of(W)[1]["losses"][0] for W in (1, 3, 4, 7)]
    assert np.allclose(first, first[0], rtol=1e-12)


def test_same_network_whatever_the_cut():
    # the flattened initial parameters are the same list of arrays for every W
    def flat(W):
        cfg = run_of(W)[0]
        return [p for st in init_params(cfg, bias_std=0.05) for layer in st for p in layer.values()]
    a = flat(1)
    for W in (3, 4, 7):
        b = flat(W)
        assert len(a) == len(b) and all(np.array_equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("W", [3, 4, 7])
def test_staleness_of_forward_passes_along_the_pipeline(W):
    # In the steady state the forward pass of mini-batch b reads, on worker s, weights that lack the updates of the
    # W - 1 - s mini-batches still in flight below it (N = 2: one mini-batch enters per worker of depth): none on the
    # last worker, W - 1 on the first.  The backward pass of b then runs on weights with all b - 1 earlier updates.
    ops = run_of(W)[1]["ops"]
    for s in range(W):
        lag = {(b - 1) - sv for (t, w, kind, b, j, sv, nv) in ops if kind == S.FWD and w == s and b > 2 * W}
        assert lag == {W - 1 - s}, (s, lag)
    for (t, w, kind, b, j, sv, nv) in ops:
        if kind == S.BWD:
            assert sv == b - 1


def test_training_converges_for_every_v_and_drifts_with_depth():
    losses = {W: np.array(run_of(W)[1]["losses"]) for W in (1, 3, 4, 7)}
    for W, l in losses.items():
        assert l[-8:].mean() < 0.6 * l[:8].mean(), "W=%d did not train" % W
    # distance of each trajectory from sequential SGD (W = 1) over the whole run: the deepest pipeline (v = 3), whose
    # forward passes are up to 6 updates behind, drifts furthest; the sequential run reaches the lowest loss
    d = {W: float(np.abs(losses[W] - losses[1]).mean()) for W in (3, 4, 7)}
    assert d[3] < d[7] and d[4] < d[7]
    assert all(losses[1][-8:].mean() < losses[W][-8:].mean() for W in (3, 4, 7))


def test_in_place_weights_stay_closer_to_sequential_sgd_than_vertical_weight_stashing():
    # The same cuts under the paper's vertical weight stashing (forward passes of later workers on the tagged, older
    # version; backward passes on the live weights): every cut still converges at this learning rate, and drifts
    # further from sequential SGD than under the in-place policy, the more so the deeper the pipeline.
    seq = np.array(run_of(1)[1]["losses"])
    for W in (3, 4, 7):
        in_place = np.array(run_of(W)[1]["losses"])
        stashed = np.array(train(W, vertical_sync=True)[1]["losses"])
        assert stashed[-8:].mean() < 0.7 * stashed[:8].mean()
        assert np.abs(stashed - seq).mean() > np.abs(in_place - seq).mean()
