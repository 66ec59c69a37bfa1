"""Shape tables of the benchmark networks, as neutral layer lists.

A network is a list of stages (the paper's workers: consecutive layers on one
accelerator, Methodology / Model Architecture); a stage is a list of layer
dicts.  Per-sample activation layout is channels-last (``[H, W, C]``) or a
flat vector ``[D]``.  Nothing here computes anything: the dicts are read by
the oracle-side tests and by the HIP binding alike.
"""
from dataclasses import dataclass, field
from typing import List, Tuple


def linear(din, dout, relu):
    return {"kind": "linear", "din": int(din), "dout": int(dout), "relu": bool(relu)}


def conv(h, w, cin, cout, r=3, stride=1, pad=1, relu=True):
    return {"kind": "conv", "h": int(h), "w": int(w), "cin": int(cin), "cout": int(cout),
            "r": int(r), "s": int(r), "stride": int(stride), "pad": int(pad), "relu": bool(relu)}


def maxpool(h, w, c, k=2, stride=2):
    return {"kind": "maxpool", "h": int(h), "w": int(w), "c": int(c), "k": int(k),
            "stride": int(stride)}


def softmax_ce(classes):
    return {"kind": "softmax_ce", "classes": int(classes)}


@dataclass
class Config:
    name: str
    dtype: str                 # "f32" or "bf16" (bf16 activations, fp32 master weights)
    M: int                     # mini-batch size
    N: int                     # micro-batches per mini-batch
    stages: List[list]         # K lists of layer dicts
    in_shape: Tuple[int, ...]  # per-sample input shape
    classes: int
    seed: int
    lr: float = 0.01
    momentum: float = 0.9
    steps: int = 20
    notes: str = ""

    @property
    def K(self):
        return len(self.stages)

    @property
    def micro(self):
        return self.M // self.N


def _tiny_mlp():
    return Config(
        name="tiny_mlp_f32", dtype="f32", M=32, N=4, seed=0, steps=20,
        in_shape=(64,), classes=10,
        stages=[[linear(64, 128, True)],
                [linear(128, 128, True), linear(128, 10, False), softmax_ce(10)]])


def _mlp_bf16():
    return Config(
        name="mlp4x1024_bf16", dtype="bf16", M=256, N=4, seed=1, steps=20,
        in_shape=(3072,), classes=10,
        stages=[[linear(3072, 1024, True)],
                [linear(1024, 1024, True)],
                [linear(1024, 1024, True)],
                [linear(1024, 1024, True), linear(1024, 10, False), softmax_ce(10)]])


def _vgg16(fc_width=4096):
    def block(h, cin, cout, n):
        layers = []
        c = cin
        for _ in range(n):
            layers.append(conv(h, h, c, cout))
            c = cout
        layers.append(maxpool(h, h, cout))
        return layers
    b1 = block(32, 3, 64, 2)
    b2 = block(16, 64, 128, 2)
    b3 = block(8, 128, 256, 3)
    b4 = block(4, 256, 512, 3)
    b5 = block(2, 512, 512, 3)
    fc = [linear(512, fc_width, True), linear(fc_width, fc_width, True),
          linear(fc_width, 10, False), softmax_ce(10)]
    return Config(
        name="vgg16_bf16", dtype="bf16", M=128, N=4, seed=2, steps=4,
        in_shape=(32, 32, 3), classes=10,
        stages=[b1 + b2, b3, b4, b5 + fc],
        notes="FC widths 512-4096-4096-10 (the 1x1x512 feature map of a 32x32 input)")


CONFIGS = {
    "tiny_mlp_f32": _tiny_mlp,
    "mlp4x1024_bf16": _mlp_bf16,
    "vgg16_bf16": _vgg16,
}


def get_config(name: str) -> Config:
    return CONFIGS[name]()


def layer_out_shape(layer, in_shape):
    """Per-sample output shape of one layer given its per-sample input shape."""
    k = layer["kind"]
    if k == "linear":
        return (layer["dout"],)
    if k == "conv":
        ho = (layer["h"] + 2 * layer["pad"] - layer["r"]) // layer["stride"] + 1
        wo = (layer["w"] + 2 * layer["pad"] - layer["s"]) // layer["stride"] + 1
        return (ho, wo, layer["cout"])
    if k == "maxpool":
        ho = (layer["h"] - layer["k"]) // layer["stride"] + 1
        wo = (layer["w"] - layer["k"]) // layer["stride"] + 1
        return (ho, wo, layer["c"])
    if k == "softmax_ce":
        return (layer["classes"],)
    raise ValueError(k)


def stage_shapes(cfg: Config):
    """[(in_shape, out_shape)] per stage, flattening [H,W,C] to [D] in front of a linear layer."""
    shapes = []
    cur = tuple(cfg.in_shape)
    for st in cfg.stages:
        s_in = cur
        for layer in st:
            cur = layer_out_shape(layer, cur)
        shapes.append((s_in, cur))
    return shapes
