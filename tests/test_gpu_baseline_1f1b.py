"""Parity of the comparison system on the GPU -- PipeDream-style 1F1B with horizontal weight stashing
(tmps_schedule_run_1f1b, tmps_backward_at) -- with the oracle's baseline (oracle/baseline.py): the task log with the
version every task read and the version every worker was at, bit for bit; losses and final weights within the dtype's
bar (for bf16 trajectories the total weight change in direction and L2 norm, as tests/test_gpu_pipeline.py)."""
import numpy as np
import pytest

from oracle import baseline
from tests.util import TOL, rel_err
from workloads import Config, get_config, init_params, make_batch
from workloads.configs import linear, softmax_ce

pytestmark = pytest.mark.gpu


def _compare(cfg, n_batches, batch, bias_std=0.05):
    from paper_2410_14312_amd import Pipeline
    tol = TOL[cfg.dtype]
    params = init_params(cfg, bias_std=bias_std)
    batches = [make_batch(cfg, i, M=batch) for i in range(n_batches)]
    ref = baseline.run_1f1b(cfg.stages, params, batches, cfg.lr, cfg.momentum,
                            precision="bf16" if cfg.dtype == "bf16" else "f64")
    pipe = Pipeline(cfg, params, baseline_1f1b=True, batch=batch)
    losses, log = pipe.run(batches)
    assert np.array_equal(log, np.array(ref["ops"], dtype=np.int32))
    assert [st.version() for st in pipe.stages] == [n_batches] * cfg.K
    # some backward pass did read an older version than its worker was at: the stashing is exercised
    assert cfg.K == 1 or np.any((log[:, 2] == 1) & (log[:, 5] < log[:, 6]))
    for i, (a, b) in enumerate(zip(losses, ref["losses"])):
        assert abs(a - b) <= tol * abs(b), "loss of batch %d: %g vs %g" % (i + 1, a, b)
    for s in range(cfg.K):
        got = pipe.get_params(s)
        for li, p in enumerate(ref["stages"][s].params):
            for k in p:
                d_g = (got[li][k].astype(np.float64) - params[s][li][k]).ravel()
                d_o = (p[k] - params[s][li][k]).ravel()
                if cfg.dtype == "f32":
                    assert rel_err(got[li][k], p[k]) < tol, (s, li, k)
                    assert rel_err(d_g, d_o) < tol, "total weight change stage %d layer %d %s" % (s, li, k)
                else:
                    if k == "w":
                        assert rel_err(got[li][k], p[k]) < tol, (s, li, k)
                    cos = float(d_g @ d_o / (np.linalg.norm(d_g) * np.linalg.norm(d_o) + 1e-300))
                    l2 = float(np.linalg.norm(d_g - d_o) / (np.linalg.norm(d_o) + 1e-300))
                    assert cos > 0.99 and l2 < 0.15, "total weight change stage %d layer %d %s: cos %g l2 %g" % (s, li, k, cos, l2)
    return pipe


def test_tiny_mlp_two_workers():
    _compare(get_config("tiny_mlp_f32"), 12, 8)


@pytest.mark.parametrize("K", [1, 3, 4])
def test_mlp_other_depths(K):
    layers = [linear(32, 32, True), linear(32, 32, True), linear(32, 32, True), linear(32, 10, False), softmax_ce(10)]
    cuts = {1: [layers], 3: [layers[:1], layers[1:3], layers[3:]], 4: [layers[:1], layers[1:2], layers[2:3], layers[3:]]}[K]
    cfg = Config(name="t", dtype="f32", M=8, N=2, stages=cuts, in_shape=(32,), classes=10, seed=3, lr=0.02)
    _compare(cfg, 14, 4)


@pytest.mark.parametrize("name", ["tiny_transformer_f32", "tiny_transformer_bf16", "tiny_resnet_f32", "tiny_resnet_bf16"])
def test_small_transformer_and_residual_networks(name):
    cfg = get_config(name)
    _compare(cfg, 8, cfg.micro)


def test_backward_at_needs_a_kept_version_and_the_run_enough_of_them():
    import torch
    from paper_2410_14312_amd import Pipeline, Stage, TmpsError
    st = Stage([linear(16, 16, True)], "f32", 4, 1, 2, 0.1, 0.9)
    st.set_params([{"w": np.eye(16, dtype=np.float32), "b": np.zeros(16, np.float32)}])
    x = torch.ones(4, 16, dtype=torch.float32, device="cuda:0")
    dy = torch.ones(4, 16, dtype=torch.float32, device="cuda:0")
    st.forward_micro(0, x)
    with pytest.raises(TmpsError) as e:
        st.backward_at(3, [0], dy=dy)           # no such version
    assert e.value.code == -1
    st.backward_at(0, [0], dy=dy)               # the live one
    st.update()
    torch.cuda.synchronize()
    cfg = get_config("tiny_mlp_f32")
    pipe = Pipeline(cfg, init_params(cfg), baseline_1f1b=True, batch=8)
    pipe.stages[0].set_shadow(0)                # the first worker keeps no older version: the run must refuse
    xs, ys = pipe.upload([make_batch(cfg, 0, M=8)] * 2)
    with pytest.raises(TmpsError) as e:
        pipe.run_device(xs, ys, 2, torch.zeros(2, dtype=torch.float32, device="cuda:0"))
    assert e.value.code == -5


def test_weight_versions_and_stash_depth_per_worker():
    # what the comparison costs in memory: worker s keeps K - s - 1 older parameter copies and K - s batches of activations
    cfg = get_config("tiny_mlp_f32")
    from paper_2410_14312_amd import Pipeline
    pipe = Pipeline(cfg, init_params(cfg), baseline_1f1b=True, batch=8)
    b0, b1 = pipe.stages[0].device_bytes(), pipe.stages[1].device_bytes()
    assert b0["kept_versions"] >= b0["params"] and b1["kept_versions"] <= 256
