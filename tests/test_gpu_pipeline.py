"""Parity of the K-stage nF1B emulator (tmps_schedule_run) with the CPU oracle's pipeline.

Integer results (task order, per-stage versions, whole-network versions) must be bit-exact.
fp32 runs: losses, final weights and the total weight change within 1e-4 (max-norm relative).
bf16 runs: losses and final weights within 2e-2.  The total weight change of a bf16 TRAJECTORY is
held to direction (cosine > 0.99) and relative L2 error < 0.15 instead: a stored activation that
falls on the other side of a bf16 rounding boundary (fp32 vs fp64 accumulation) perturbs later
layers, after a few layers the two runs round independently, and a weight gradient -- a sum with
both signs over the mini-batch -- amplifies that rounding noise by its cancellation factor
(tests/test_oracle_precision.py measures 9 % between the exact and the bf16-policy oracle).  The
element-by-element 2e-2 bar on identical inputs is held per stage step in tests/test_gpu_stage.py,
including every stage of the benchmark configurations at full size.
"""
import numpy as np
import pytest

from oracle import pipeline
from tests.util import TOL, rel_err
from workloads import Config, get_config, init_params, make_batch
from workloads.configs import conv, linear, maxpool, softmax_ce

pytestmark = pytest.mark.gpu


def _compare(cfg, n_steps, loss_tol=None, bias_std=0.0, vertical_sync=False):
    import torch
    from paper_2410_14312_amd import Pipeline
    tol = TOL[cfg.dtype]
    params = init_params(cfg, bias_std=bias_std)
    batches = [make_batch(cfg, i) for i in range(n_steps)]
    ref = pipeline.run(cfg, params, batches, vertical_sync=vertical_sync)
    pipe = Pipeline(cfg, params, vertical_sync=vertical_sync)
    losses, log = pipe.run(batches)
    # integer bookkeeping: bit-exact
    assert np.array_equal(log, np.array(ref["ops"], dtype=np.int32))
    assert [st.version() for st in pipe.stages] == [n_steps] * cfg.K
    lt = tol if loss_tol is None else loss_tol
    for i, (a, b) in enumerate(zip(losses, ref["losses"])):
        assert abs(a - b) <= lt * abs(b), "loss of mini-batch %d: %g vs %g" % (i + 1, a, b)
    for s in range(cfg.K):
        got = pipe.get_params(s)
        for li, p in enumerate(ref["stages"][s].params):
            for k in p:
                d_g = (got[li][k].astype(np.float64) - params[s][li][k]).ravel()
                d_o = (p[k] - params[s][li][k]).ravel()
                if cfg.dtype == "f32":
                    assert rel_err(got[li][k], p[k]) < tol, (s, li, k)
                    e = rel_err(d_g, d_o)
                    assert e < tol, "total weight change stage %d layer %d %s: %g" % (s, li, k, e)
                else:
                    if k == "w":
                        assert rel_err(got[li][k], p[k]) < tol, (s, li, k)
                    cos = float(d_g @ d_o / (np.linalg.norm(d_g) * np.linalg.norm(d_o) + 1e-300))
                    l2 = float(np.linalg.norm(d_g - d_o) / (np.linalg.norm(d_o) + 1e-300))
                    assert cos > 0.99 and l2 < 0.15, "total weight change stage %d layer %d %s: cos %g l2 %g" % (s, li, k, cos, l2)
    return losses


def test_tiny_mlp_f32_20_steps():
    cfg = get_config("tiny_mlp_f32")
    losses = _compare(cfg, cfg.steps)
    assert np.mean(losses[-5:]) < np.mean(losses[:5])


def test_tiny_mlp_f32_other_pipeline_depths():
    base = get_config("tiny_mlp_f32")
    layers = [l for st in base.stages for l in st]
    for stages in ([layers], [layers[:1], layers[1:2], layers[2:]]):
        cfg = Config(name="t", dtype="f32", M=32, N=4, stages=stages, in_shape=(64,), classes=10, seed=0)
        _compare(cfg, 8, bias_std=0.05)


def test_mlp_bf16_trajectory():
    cfg = get_config("mlp4x1024_bf16")
    _compare(cfg, 6)


def test_v_greater_than_one_schedule_runs_and_logs():
    # W=4 stages with N=2 micro-batches: two interleaved update sequences (version difference 2)
    layers = [linear(32, 32, True), linear(32, 32, True), linear(32, 32, True), linear(32, 10, False), softmax_ce(10)]
    cfg = Config(name="t", dtype="f32", M=8, N=2, stages=[layers[:1], layers[1:2], layers[2:3], layers[3:]],
                 in_shape=(32,), classes=10, seed=3)
    _compare(cfg, 9, bias_std=0.05)


def test_version_difference_three_on_seven_streams():
    # W=7 stages, N=2: three interleaved update sequences; the forward passes of worker 0 run on weights 6 updates old
    layers = [linear(32, 32, True) for _ in range(6)] + [linear(32, 10, False), softmax_ce(10)]
    stages = [[l] for l in layers[:6]] + [layers[6:]]
    cfg = Config(name="t", dtype="f32", M=8, N=2, stages=stages, in_shape=(32,), classes=10, seed=11, lr=0.005)
    from paper_2410_14312_amd import version_diff_simulated
    assert version_diff_simulated(7, 2) == 3
    _compare(cfg, 24, bias_std=0.05)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_conv_net_three_stages(dtype):
    stages = [[conv(8, 8, 3, 16), conv(8, 8, 16, 16), maxpool(8, 8, 16)],
              [conv(4, 4, 16, 32), maxpool(4, 4, 32)],
              [linear(2 * 2 * 32, 64, True), linear(64, 10, False), softmax_ce(10)]]
    cfg = Config(name="t", dtype=dtype, M=16, N=4, stages=stages, in_shape=(8, 8, 3), classes=10, seed=7)
    _compare(cfg, 5, bias_std=0.05)


@pytest.mark.parametrize("name", ["tiny_transformer_f32", "tiny_transformer_bf16", "tiny_resnet_f32", "tiny_resnet_bf16"])
def test_small_transformer_and_residual_networks(name):
    cfg = get_config(name)
    _compare(cfg, 5, bias_std=0.05)


def test_vgg16_bf16_two_steps():
    cfg = get_config("vgg16_bf16")
    _compare(cfg, 2)


def test_run_rejects_small_stash_and_mismatched_stages():
    import ctypes as C
    import torch
    from paper_2410_14312_amd import Stage, TmpsError, lib
    from paper_2410_14312_amd.binding import _check
    a = Stage([linear(16, 16, True)], "f32", 4, 2, 2, 0.1, 0.9)                      # one group only
    b = Stage([linear(16, 10, False), softmax_ce(10)], "f32", 4, 2, 2, 0.1, 0.9, borrow_input=True)
    x = torch.zeros(16, 16, dtype=torch.float32, device="cuda:0")
    y = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    losses = torch.zeros(2, dtype=torch.float32, device="cuda:0")
    handles = (C.c_void_p * 2)(a.handle, b.handle)
    streams = (C.c_void_p * 2)(0, 0)
    with pytest.raises(TmpsError) as e:
        _check(lib().tmps_schedule_run(handles, 2, 2, 2, x.data_ptr(), y.data_ptr(), streams, losses.data_ptr(), None))
    assert e.value.code == -5
    with pytest.raises(TmpsError) as e:
        _check(lib().tmps_schedule_run(handles, 2, 4, 2, x.data_ptr(), y.data_ptr(), streams, losses.data_ptr(), None))
    assert e.value.code == -3


@pytest.mark.parametrize("name", ["tiny_mlp_f32", "tiny_transformer_bf16"])
def test_resume_from_stage_checkpoints(name, tmp_path):
    """Section "Checkpointing": a pipeline restored from the files every stage wrote at the end of an epoch goes on
    exactly (bit for bit) as the pipeline that wrote them, and a damaged file of one stage pulls all stages back."""
    import torch
    from paper_2410_14312_amd import Pipeline, checkpoint
    cfg = get_config(name)
    params = init_params(cfg, bias_std=0.05)
    batches = [make_batch(cfg, i) for i in range(9)]
    d = str(tmp_path)
    a = Pipeline(cfg, params)
    a.run(batches[:3]); a.save_checkpoint(d, 1)
    a.run(batches[3:6]); a.save_checkpoint(d, 2)
    losses_a, _ = a.run(batches[6:])
    # resume in a new pipeline from epoch 2 and train the third epoch
    b = Pipeline(cfg, params)
    assert b.resume(d) == 2
    assert [st.version() for st in b.stages] == [6] * cfg.K
    losses_b, log_b = b.run(batches[6:])
    assert losses_b == losses_a
    assert [st.version() for st in b.stages] == [9] * cfg.K
    # the version log counts from the run's start, as the plan and the oracle's resumed run do
    from paper_2410_14312_amd import schedule_plan
    assert np.array_equal(log_b, schedule_plan(cfg.K, cfg.N, 3))
    for s in range(cfg.K):
        for pa, pb in zip(a.get_params(s), b.get_params(s)):
            for k in pa:
                assert np.array_equal(pa[k], pb[k]), (s, k)
        for ma, mb in zip(a.stages[s].get_momentum(), b.stages[s].get_momentum()):
            for k in ma:
                assert np.array_equal(ma[k], mb[k]), (s, k)
    # stage 1's epoch-2 file is cut short: every stage goes back to epoch 1
    path = checkpoint.stage_file(d, cfg.K - 1, 2)
    data = open(path, "rb").read()
    open(path, "wb").write(data[:len(data) // 2])
    c = Pipeline(cfg, params)
    assert c.resume(d) == 1
    assert [st.version() for st in c.stages] == [3] * cfg.K
    c.run(batches[3:6])
    losses_c, _ = c.run(batches[6:])
    assert losses_c == losses_a
    # nothing to resume from
    assert Pipeline(cfg, params).resume(str(tmp_path / "empty")) is None


def test_vertical_weight_stashing_on_the_tiny_mlp():
    """The paper's own weight policy for forward passes (vertical weight stashing): parity with the oracle in that
    mode, and a different trajectory from the in-place mode once a later worker runs ahead of worker 1."""
    cfg = get_config("tiny_mlp_f32")
    vs = _compare(cfg, 12, vertical_sync=True)
    ip = _compare(cfg, 12)
    assert vs[0] == ip[0] and vs != ip


@pytest.mark.parametrize("name", ["tiny_transformer_f32", "tiny_transformer_bf16", "tiny_resnet_bf16"])
def test_vertical_weight_stashing_small_networks(name):
    _compare(get_config(name), 5, bias_std=0.05, vertical_sync=True)


def test_vertical_weight_stashing_deep_pipeline_and_errors():
    # W=4, N=2: the last worker runs up to 3 versions ahead of the tag
    from paper_2410_14312_amd import Pipeline, TmpsError, schedule_shadow_versions
    layers = [linear(32, 32, True), linear(32, 32, True), linear(32, 32, True), linear(32, 10, False), softmax_ce(10)]
    cfg = Config(name="t", dtype="f32", M=8, N=2, stages=[layers[:1], layers[1:2], layers[2:3], layers[3:]],
                 in_shape=(32,), classes=10, seed=3)
    assert [schedule_shadow_versions(4, 2, s) for s in range(4)] == [0, 1, 2, 3]
    assert [schedule_shadow_versions(4, 8, s) for s in range(4)] == [0, 1, 1, 1]
    _compare(cfg, 10, bias_std=0.05, vertical_sync=True)
    # a stage that keeps too few versions is refused before anything runs
    pipe = Pipeline(cfg, init_params(cfg, bias_std=0.05), vertical_sync=True)
    pipe.stages[3].set_shadow(1)
    with pytest.raises(TmpsError):
        pipe.run([make_batch(cfg, i) for i in range(3)])
    # a version that is not kept is an error of the versioned forward call
    import torch
    st = pipe.stages[0]
    x = st.prepare_input(make_batch(cfg, 0)[0][:cfg.micro])
    with pytest.raises(TmpsError):
        st.forward_micro_at(5, 0, x)


def test_second_run_and_failed_run_on_the_same_stages():
    """A second tmps_schedule_run on the same stages logs the same numbers as the plan (versions count from the run's
    start) and continues the oracle's trajectory; a run is refused while a stage still holds a forwarded micro-batch."""
    import torch
    from paper_2410_14312_amd import Pipeline, TmpsError, schedule_plan
    cfg = get_config("tiny_mlp_f32")
    params = init_params(cfg)
    batches = [make_batch(cfg, i) for i in range(6)]
    ref = pipeline.run(cfg, params, batches)
    pipe = Pipeline(cfg, params)
    l1, log1 = pipe.run(batches[:3])
    l2, log2 = pipe.run(batches[3:])
    plan = schedule_plan(cfg.K, cfg.N, 3)
    assert np.array_equal(log1, plan) and np.array_equal(log2, plan)
    assert [st.version() for st in pipe.stages] == [6] * cfg.K
    # the two runs drain the pipeline in between, so their trajectory is that of two oracle runs in a row
    mid = pipeline.run(cfg, params, batches[:3])
    ref2 = pipeline.run(cfg, [[dict(p) for p in st.params] for st in mid["stages"]], batches[3:],
                        momentum=[st.bufs for st in mid["stages"]], versions=[3] * cfg.K)
    for a, b in zip(l1 + l2, mid["losses"] + ref2["losses"]):
        assert abs(a - b) <= 1e-4 * abs(b)
    del ref
    # a run is refused while a stage holds a forwarded micro-batch, and runs again once that mini-batch is done
    x, y = pipe.upload(batches[:2])
    losses = torch.zeros(2, dtype=torch.float32, device=pipe.device)
    last = pipe.stages[1]
    xin = torch.zeros(cfg.M, last.in_elems, dtype=torch.float32, device=pipe.device)
    last.forward_micro(0, xin[:cfg.micro], labels=y[:cfg.micro])
    with pytest.raises(TmpsError) as e:
        pipe.run_device(x, y, 2, losses)
    assert e.value.code == -4
    torch.cuda.synchronize()
    for j in range(1, cfg.N):
        last.forward_micro(j, xin[j * cfg.micro:(j + 1) * cfg.micro], labels=y[j * cfg.micro:(j + 1) * cfg.micro])
    last.backward(list(range(cfg.N)), dx=torch.empty(cfg.M * last.in_elems, dtype=torch.float32, device=pipe.device))
    torch.cuda.synchronize()
    log3 = pipe.run_device(x, y, 2, losses)
    assert np.array_equal(log3, schedule_plan(cfg.K, cfg.N, 2))
