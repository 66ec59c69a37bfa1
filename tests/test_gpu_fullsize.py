"""Stage steps of the two large benchmark configurations at their real layer shapes, HIP path against the CPU
oracle element by element (tests/test_gpu_stage.py holds the small shapes and the MLP / VGG configurations at
full size).

The oracle needs tens of seconds for a whole mini-batch of these stages, so only one stage of each network runs
with the configuration's own mini-batch (M, N): the inner transformer stage and the last residual stage (with
pooling, classifier and loss).  The other stages run with the configuration's micro-batch size, so every
forward launch has the shape the benchmark times, but with N = 2 micro-batches per mini-batch, so the backward
pass covers 2 micro-batches instead of 8.  The residual stages are tens of ReLU layers deep: see `deep` in
tests/test_gpu_stage.py for the bar they are held to in bf16; one of them is also run with fp32 storage, to the
full element-wise bar.
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
                   borrow=stage > 0, deep=True)


@pytest.mark.parametrize("stage", [2, 3])
def test_resnet50_stage_in_fp32(stage):
    # the same layer graphs and sizes (the deepest stage, six blocks, and the last one) with fp32 storage, where
    # rounding ties are rare: the element-wise bar on all but a handful of elements (`deep` in tests/test_gpu_stage.py)
    from workloads import get_config
    cfg = get_config("resnet50_bf16")
    run_stage_case(cfg.stages[stage], "f32", cfg.micro, 2, seed=503, borrow=True, deep=True)
