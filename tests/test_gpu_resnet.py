"""Parity of the residual-network stage kernels (per-channel affine, residual join with identity and
projection shortcuts, padded max pooling, global average pooling, gradients of a result that several layers
read) with the CPU oracle, through the C ABI, with the stage harness of tests/test_gpu_stage.py.
"""
import numpy as np
import pytest

from tests.test_gpu_stage import run_stage_case
from workloads.configs import affine, avgpool, bottleneck, conv, linear, maxpool, softmax_ce

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,cin,cout,relu,micro,N", [(6, 8, 16, True, 3, 2), (9, 16, 24, False, 2, 2), (14, 8, 72, True, 5, 2)])
def test_conv_affine_stage(dtype, h, cin, cout, relu, micro, N):
    specs = [conv(h, h, cin, cout, 3, 1, 1, False), affine(h, h, cout, relu), conv(h, h, cout, 8, 1, 1, 0, True)]
    run_stage_case(specs, dtype, micro, N, seed=h + cout)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stem_stage(dtype):
    # 7x7 stride-2 convolution on 3 channels, affine + ReLU, 3x3 stride-2 max pooling with padding 1
    specs = [conv(20, 20, 3, 16, 7, 2, 3, False), affine(10, 10, 16, True), maxpool(10, 10, 16, 3, 2, 1), conv(5, 5, 16, 8, 1, 1, 0, True)]
    run_stage_case(specs, dtype, 3, 2, seed=51, has_pool=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,cin,width,stride,project", [
    (8, 32, 8, 1, False),    # identity shortcut: the stage input is read by the first convolution and by the join
    (8, 16, 8, 1, True),     # projection shortcut, stride 1
    (8, 16, 8, 2, True),     # projection shortcut, stride 2 on the 3x3 and on the projection
    (7, 24, 16, 2, True),    # odd size, ragged channel counts
])
def test_bottleneck_stage(dtype, h, cin, width, stride, project):
    layers, ho, cout = bottleneck(h, cin, width, stride, project)
    run_stage_case(layers, dtype, 3, 2, seed=h * 10 + cin + stride)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_bottlenecks_inside_a_stage(dtype):
    # the join of the first block is read by the second block's first convolution and by its join
    b1, h, c = bottleneck(6, 16, 8, 1, True)
    b2, h, c = bottleneck(h, c, 8, 1, False)
    run_stage_case([conv(6, 6, 8, 16, 3, 1, 1, True)] + b1 + b2, dtype, 2, 3, seed=61)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("borrow", [False, True])
def test_block_avgpool_classifier_stage(dtype, borrow):
    b1, h, c = bottleneck(4, 16, 8, 2, True)
    specs = b1 + [avgpool(h, h, c), linear(c, 10, False), softmax_ce(10)]
    run_stage_case(specs, dtype, 4, 2, seed=71, borrow=borrow)


@pytest.mark.parametrize("name,stage", [("tiny_resnet_f32", 0), ("tiny_resnet_f32", 1),
                                        ("tiny_resnet_bf16", 0), ("tiny_resnet_bf16", 1)])
def test_tiny_resnet_config_stage(name, stage):
    from workloads import get_config
    cfg = get_config(name)
    run_stage_case(cfg.stages[stage], cfg.dtype, cfg.micro, cfg.N, seed=300 + stage, has_pool=stage == 0, borrow=stage > 0)
