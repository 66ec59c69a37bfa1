"""The FLOP accounting of bench.py (what its MFMA fractions are computed from) against counts written out by hand
from the layer shapes of the benchmark configurations, and the per-stage split against the whole."""
import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import bench  # noqa: E402
from workloads import get_config  # noqa: E402

NAMES = ("tiny_mlp_f32", "mlp4x1024_bf16", "vgg16_bf16", "resnet50_bf16", "gpt2_small_bf16")


def forward_macs_per_sample(cfg):
    w = bench.algorithmic_work(cfg)
    return sum(v[1] for k, v in w.items() if k.endswith("_fwd")) / 2.0 / cfg.M


def test_tiny_mlp_forward_macs():
    # 64-128-128-10
    assert forward_macs_per_sample(get_config("tiny_mlp_f32")) == 64 * 128 + 128 * 128 + 128 * 10


def test_mlp_forward_macs():
    # 3072-1024-1024-1024-1024-10
    assert forward_macs_per_sample(get_config("mlp4x1024_bf16")) == 3072 * 1024 + 3 * 1024 * 1024 + 1024 * 10


def test_vgg16_forward_macs():
    # 13 3x3 convolutions on 32x32 images (channels 64,64 | 128,128 | 256 x3 | 512 x3 | 512 x3, a 2x2 pooling after each
    # block) and the 512-4096-4096-10 classifier
    macs, hw, cin = 0, 32, 3
    for block in ((64, 64), (128, 128), (256, 256, 256), (512, 512, 512), (512, 512, 512)):
        for cout in block:
            macs += hw * hw * 9 * cin * cout
            cin = cout
        hw //= 2
    macs += 512 * 4096 + 4096 * 4096 + 4096 * 10
    assert forward_macs_per_sample(get_config("vgg16_bf16")) == macs


def test_resnet50_forward_macs():
    # stem 7x7/2 to 112x112x64, then bottleneck groups of 3/4/6/3 blocks (widths 64/128/256/512, outputs 4x as wide,
    # stride on the 3x3 convolution of a group's first block, projection shortcut on that block), 1000-way classifier
    macs = 112 * 112 * 49 * 3 * 64
    hw, cin = 56, 64
    for gi, (blocks, width) in enumerate(((3, 64), (4, 128), (6, 256), (3, 512))):
        for b in range(blocks):
            stride = 2 if (b == 0 and gi > 0) else 1
            out_hw = hw // stride
            macs += hw * hw * cin * width                       # 1x1 reduce, at the input resolution
            macs += out_hw * out_hw * 9 * width * width         # 3x3, carries the stride
            macs += out_hw * out_hw * width * 4 * width         # 1x1 expand
            if b == 0:
                macs += out_hw * out_hw * cin * 4 * width       # projection shortcut
            cin, hw = 4 * width, out_hw
    macs += 2048 * 1000
    got = forward_macs_per_sample(get_config("resnet50_bf16"))
    assert got == macs
    assert abs(got - 4.09e9) < 0.01 * 4.09e9                    # the usual figure for this network at 224x224


def test_gpt2_forward_macs():
    # per token and layer: d x 3d, d x d, d x 4d, 4d x d; causal attention: a query at position i sees i + 1 keys,
    # two products of the head size per (query, key) pair; output layer d x vocabulary
    d, layers, s, vocab = 768, 12, 512, 32000
    linear = layers * (d * 3 * d + d * d + 2 * d * 4 * d) + d * vocab
    attention = layers * 2 * d * (s + 1) / 2.0
    assert forward_macs_per_sample(get_config("gpt2_small_bf16")) == pytest.approx((linear + attention) * s, rel=1e-12)


@pytest.mark.parametrize("name", NAMES)
def test_stages_add_up_to_the_whole(name):
    cfg = get_config(name)
    whole = bench.algorithmic_work(cfg)
    parts = [bench.algorithmic_work(cfg, only_stage=s) for s in range(cfg.K)]
    for klass, (launches, flops, nbytes) in whole.items():
        assert sum(p.get(klass, [0, 0.0, 0.0])[0] for p in parts) == launches
        assert sum(p.get(klass, [0, 0.0, 0.0])[1] for p in parts) == pytest.approx(flops, rel=1e-12)
        assert sum(p.get(klass, [0, 0.0, 0.0])[2] for p in parts) == pytest.approx(nbytes, rel=1e-12)


@pytest.mark.parametrize("name", NAMES[1:])
def test_training_flops_are_three_forward_passes_minus_the_first_input_gradient(name):
    cfg = get_config(name)
    w = bench.algorithmic_work(cfg)
    fwd = sum(v[1] for k, v in w.items() if k in ("dense_fwd", "conv_fwd"))
    dgrad = sum(v[1] for k, v in w.items() if k in ("dense_dgrad", "conv_dgrad"))
    wgrad = sum(v[1] for k, v in w.items() if k in ("dense_wgrad", "conv_wgrad"))
    assert wgrad == pytest.approx(fwd, rel=1e-12)
    if name == "gpt2_small_bf16":
        assert dgrad == pytest.approx(fwd, rel=1e-12)   # its first layer is an embedding: every contraction has an input gradient
    else:
        assert dgrad < fwd                              # the first layer has no input gradient
        assert dgrad > 0.9 * fwd or name == "mlp4x1024_bf16"   # (the MLP's first layer is half of its work)
