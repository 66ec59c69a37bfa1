"""Stage steps of the two large benchmark configurations at their real layer shapes, HIP path against the CPU
oracle element by element (tests/test_gpu_stage.py holds the small shapes and the MLP / VGG configurations at
full size).

The oracle needs tens of seconds for a whole mini-batch of these stages, so only one stage of each network runs
with the configuration's own mini-batch (M, N): the inner transformer stage and the last residual stage (with
pooling, classifier and loss).  The other stages run with the configuration's micro-batch size, so every
forward launch has the shape the benchmark times, but with N = 2 micro-batches per mini-batch, so the backward
pass covers 2 micro-batches instead of 8.  The residual stages are tens of ReLU layers deep: see `deep` in
tests/test_gpu_stage.py for the bar whole stages are held to in bf16 (tests/test_gpu_resnet50_blocks.py holds every
block of them to the element-wise bar); two of them are also run with fp32 storage.
"""
import pytest

from tests.test_gpu_stage import run_stage_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("stage,full", [(1, True), (0, False), (3, False)])
def test_gpt2_small_stage(stage, full):
    from workloads import get_config
    cfg = get_config("gpt2_small_bf16")
    run_stage_case(cfg.stages[stage], cfg.dtype, cfg.micro, cfg.N if full else 2, seed=400 + stage, borrow=stage > 0)


@pytest.mark.parametrize("stage,full", [(3, True), (0, False), (1, False), (2, False)])
def test_resnet50_stage(stage, full):
    from workloads import get_config
    cfg = get_config("resnet50_bf16")
    run_stage_case(cfg.stages[stage], cfg.dtype, cfg.micro, cfg.N if full else 2, seed=500 + stage, has_pool=stage == 0,
                   borrow=stage > 0, deep=True, deep_l2=(0.04, 0.1, 0.2, 0.1)[stage])


@pytest.mark.parametrize("stage", [2, 3])
def test_resnet50_stage_in_fp32(stage):
    # the same layer graphs and sizes (the deepest stage, six blocks, and the last one) with fp32 storage, where
    # rounding ties are rare: the element-wise bar on all but a handful of elements (`deep` in tests/test_gpu_stage.py)
    from workloads import get_config
    cfg = get_config("resnet50_bf16")
    run_stage_case(cfg.stages[stage], "f32", cfg.micro, 2, seed=503, borrow=True, deep=True)


@pytest.mark.parametrize("name", ["gpt2_small_bf16", "resnet50_bf16"])
def test_benchmark_launch_configuration_at_full_size(name):
    """The whole pipeline in the configuration bench.py times (K stages on K streams, host threads issuing), at full
    size, held by properties that need no oracle run of that size: overlapping the stages changes no number (every
    loss, every parameter and the version log equal those of the same run with all workers on ONE stream, bit for
    bit, and those of a second K-stream run), the version log is the planned one, every loss is finite and the first
    loss of the language model is that of an untrained one.  Each stage's step is held to the oracle element by
    element by the tests above."""
    import numpy as np
    from paper_2410_14312_amd import Pipeline, schedule_plan
    from workloads import get_config, init_params, make_batch
    cfg = get_config(name)
    params = init_params(cfg)
    batches = [make_batch(cfg, i % 2) for i in range(6)]
    runs = []
    for one_stream in (False, True, False):
        pipe = Pipeline(cfg, params, one_stream=one_stream)
        losses, log = pipe.run(batches)
        runs.append((losses, log, [pipe.get_params(s) for s in range(cfg.K)]))
        del pipe
    plan = np.array(schedule_plan(cfg.K, cfg.N, len(batches)), dtype=np.int32).reshape(-1, 7)
    for losses, log, weights in runs:
        assert np.array_equal(log, plan)
        assert all(np.isfinite(losses))
    for other in runs[1:]:
        assert other[0] == runs[0][0]
        for sa, sb in zip(runs[0][2], other[2]):
            for pa, pb in zip(sa, sb):
                for k in pa:
                    assert np.array_equal(pa[k], pb[k])
    if name.startswith("gpt2"):
        # an untrained language model with small initial logits: the loss of the first mini-batch is ln(vocabulary)
        assert abs(runs[0][0][0] - np.log(cfg.classes)) < 0.1 * np.log(cfg.classes)


def test_gpt2_small_pipeline_against_the_oracle():
    """The configuration bench.py times -- GPT-2-small, K = 4 stages on 4 streams, N = 8 micro-batches -- for two
    mini-batches against the oracle's pipeline at full size: the version log bit for bit, both losses and the final
    weights within the bf16 bar, the total weight change of every tensor in direction and L2 norm (section "Work
    Scheduling"; update rule of TiMePReSt).  The second mini-batch's forward passes already run on updated weights
    of the later stages, and its backward passes on the weights after the first update."""
    from tests.test_gpu_pipeline import _compare
    from workloads import get_config
    cfg = get_config("gpt2_small_bf16")
    losses = _compare(cfg, 2)
    assert all(l == l for l in losses)
