"""Vertical weight stashing in the oracle (Methodology, first paragraph; "GPU Memory Overhead").

The paper keeps every forward pass on ONE weight version across the workers: a micro-batch is tagged when it enters
worker 1, and later workers, which may have applied newer updates by the time it reaches them, run it on the version
with that tag, kept aside until no forward pass needs it.  Pins:

* consistency: the logits of every micro-batch equal those of the WHOLE network evaluated in one piece on the weights
  all workers had after nv updates, nv being the tag in the schedule log;
* with one worker there is nothing to stash: identical to the in-place run;
* worker 1 always reads its live weights (the tag is its own version), later workers read older ones exactly when the
  log says they are ahead, and then the two policies give different numbers;
* the number of older versions a worker must keep: none on worker 1, one per later worker for the benchmark's
  W = 4, N = 8, growing with depth when N is small.
"""
import numpy as np
import pytest

from oracle import pipeline
from oracle import schedule as S
from oracle.stage import Stage
from workloads import Config, get_config, init_params, make_batch
from workloads.configs import linear, softmax_ce


def _cfg(W, N=2, M=8):
    layers = [linear(16, 16, True) for _ in range(W - 1)] + [linear(16, 10, False), softmax_ce(10)]
    stages = [[l] for l in layers[:W - 1]] + [layers[W - 1:]]
    return Config(name="vs", dtype="f32", M=M, N=N, stages=stages, in_shape=(16,), classes=10, seed=5, lr=0.05)


def _run_with_snapshots(cfg, n, vertical_sync):
    """Pipeline run that also records every worker's parameters after each of its updates."""
    snaps = {}
    orig = Stage.update

    def recording(self):
        orig(self)
        snaps.setdefault(id(self), {})[self.version] = [{k: v.copy() for k, v in p.items()} for p in self.params]

    Stage.update = recording
    try:
        params = init_params(cfg, bias_std=0.05)
        batches = [make_batch(cfg, i) for i in range(n)]
        trace = {}
        res = pipeline.run(cfg, params, batches, trace=trace, vertical_sync=vertical_sync)
    finally:
        Stage.update = orig
    per_stage = []
    for s, st in enumerate(res["stages"]):
        h = dict(snaps.get(id(st), {}))
        h[0] = [{k: np.asarray(v, dtype=np.float64) for k, v in p.items()} for p in params[s]]
        per_stage.append(h)
    return res, trace, per_stage, batches


@pytest.mark.parametrize("W,N", [(2, 4), (3, 2), (4, 2), (4, 4)])
def test_every_forward_pass_sees_one_version_of_the_whole_network(W, N):
    cfg = _cfg(W, N, M=4 * N)
    res, trace, hist, batches = _run_with_snapshots(cfg, 3 * W + 2, vertical_sync=True)
    micro = cfg.M // cfg.N
    all_specs = [sp for st in cfg.stages for sp in st]
    checked = 0
    for (t, s, kind, b, j, sv, nv) in res["ops"]:
        if kind != S.FWD or s != W - 1:
            continue
        whole = [p for st in range(W) for p in hist[st][nv]]
        net = Stage(all_specs, whole, cfg.lr, cfg.momentum, cfg.M, cfg.N)
        x, y = batches[b - 1]
        logits, _ = net.forward_micro(0, x[j * micro:(j + 1) * micro], y[j * micro:(j + 1) * micro])
        assert np.allclose(trace[("F", b, j, s)], logits, rtol=1e-12, atol=1e-12), (b, j, nv)
        checked += 1
    assert checked == (3 * W + 2) * N


def test_in_place_run_is_not_version_consistent_once_a_worker_is_ahead():
    cfg = _cfg(3, 2)
    res, trace, hist, batches = _run_with_snapshots(cfg, 10, vertical_sync=False)
    micro = cfg.M // cfg.N
    all_specs = [sp for st in cfg.stages for sp in st]
    differs = 0
    for (t, s, kind, b, j, sv, nv) in res["ops"]:
        if kind == S.FWD and s == 2 and sv > nv:
            whole = [p for st in range(3) for p in hist[st][nv]]
            net = Stage(all_specs, whole, cfg.lr, cfg.momentum, cfg.M, cfg.N)
            x, y = batches[b - 1]
            logits, _ = net.forward_micro(0, x[j * micro:(j + 1) * micro], y[j * micro:(j + 1) * micro])
            differs += int(not np.allclose(trace[("F", b, j, s)], logits, rtol=1e-9))
    assert differs > 0


def test_single_worker_has_nothing_to_stash():
    base = get_config("tiny_mlp_f32")
    layers = [l for st in base.stages for l in st]
    cfg = Config(name="t", dtype="f32", M=32, N=4, stages=[layers], in_shape=(64,), classes=10, seed=0)
    params = init_params(cfg)
    batches = [make_batch(cfg, i) for i in range(5)]
    a = pipeline.run(cfg, params, batches)
    b = pipeline.run(cfg, params, batches, vertical_sync=True)
    assert a["losses"] == b["losses"]
    assert b["stages"][0].keep_versions == 0


def test_policies_agree_until_a_later_worker_is_ahead_and_differ_after():
    cfg = _cfg(3, 2)
    params = init_params(cfg, bias_std=0.05)
    batches = [make_batch(cfg, i) for i in range(10)]
    ta, tb = {}, {}
    a = pipeline.run(cfg, params, batches, trace=ta)
    b = pipeline.run(cfg, params, batches, trace=tb, vertical_sync=True)
    first_ahead = min(bb for (t, s, kind, bb, j, sv, nv) in a["ops"] if kind == S.FWD and sv > nv)
    for bb in range(1, first_ahead):
        assert a["losses"][bb - 1] == b["losses"][bb - 1]
    assert a["losses"][first_ahead - 1] != b["losses"][first_ahead - 1]
    # worker 1 reads its live weights under both policies: its version IS the tag
    for (t, s, kind, bb, j, sv, nv) in a["ops"]:
        if kind == S.FWD and s == 0:
            assert sv == nv


@pytest.mark.parametrize("W,N,need", [(2, 4, [0, 1]), (4, 8, [0, 1, 1, 1]), (4, 4, [0, 1, 1, 2]), (4, 2, [0, 1, 2, 3])])
def test_versions_a_worker_keeps(W, N, need):
    cfg = _cfg(W, N, M=2 * N)
    params = init_params(cfg)
    res = pipeline.run(cfg, params, [make_batch(cfg, i % 3) for i in range(4 * W)], vertical_sync=True)
    assert [st.keep_versions for st in res["stages"]] == need
    assert all(len(st.history) <= st.keep_versions for st in res["stages"])   # superseded versions are dropped
