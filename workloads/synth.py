"""Seeded synthetic inputs, labels and initial parameters.

Inputs follow the recipe of the benchmark configurations: standard-normal
inputs, labels uniform over the classes, He-normal weights ``N(0, 2/fan_in)``
and zero biases; layer-normalisation and per-channel affine gains 1 and shifts 0; embedding tables
``N(0, 0.02^2)``; token inputs uniform over the vocabulary, S+1 per sample
(the first S are the input, the last S the next-token targets).  Everything is drawn with numpy's PCG64 generator keyed by
``(seed, stream, index)`` so that a batch can be regenerated independently.
The only numeric helper is ``to_bf16_grid``, which snaps fp32 *input data* to
values exactly representable in bfloat16 so that both implementations start
from identical numbers; it is data preparation, not part of the method.
"""
import numpy as np


def _rng(seed, stream, index=0):
    return np.random.default_rng([int(seed), int(stream), int(index)])


def to_bf16_grid(a):
    """Round fp32 values to the nearest (ties-to-even) bfloat16-representable value, returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def fan_in(layer):
    if layer["kind"] == "linear":
        return layer["din"]
    if layer["kind"] == "conv":
        return layer["r"] * layer["s"] * layer["cin"]
    raise ValueError(layer["kind"])


def param_shapes(layer):
    """{'w': shape, 'b': shape} for layers with parameters, else {}."""
    if layer["kind"] == "linear":
        return {"w": (layer["dout"], layer["din"]), "b": (layer["dout"],)}
    if layer["kind"] == "conv":
        return {"w": (layer["cout"], layer["r"], layer["s"], layer["cin"]), "b": (layer["cout"],)}
    if layer["kind"] == "layernorm":      # w = gain, b = shift
        return {"w": (layer["d"],), "b": (layer["d"],)}
    if layer["kind"] == "affine":         # w = gain, b = shift, per channel
        return {"w": (layer["c"],), "b": (layer["c"],)}
    if layer["kind"] == "embedding":      # w = token table, b = position table
        return {"w": (layer["vocab"], layer["d"]), "b": (layer["s"], layer["d"])}
    return {}


def init_params(cfg, bias_std=0.0):
    """Initial parameters: list (stages) of list (layers) of dicts of fp32 arrays."""
    out = []
    idx = 0
    for st in cfg.stages:
        ps = []
        for layer in st:
            shp = param_shapes(layer)
            p = {}
            if shp and layer["kind"] in ("layernorm", "affine"):
                g = _rng(cfg.seed, 1, idx)
                p["w"] = np.full(shp["w"], layer.get("init_gain", 1.0), dtype=np.float32)
                p["b"] = np.zeros(shp["b"], dtype=np.float32)
                if bias_std > 0.0:
                    p["w"] += (g.standard_normal(shp["w"]) * bias_std).astype(np.float32)
                    p["b"] += (g.standard_normal(shp["b"]) * bias_std).astype(np.float32)
            elif shp and layer["kind"] == "embedding":
                g = _rng(cfg.seed, 1, idx)
                p["w"] = (g.standard_normal(shp["w"]) * 0.02).astype(np.float32)
                p["b"] = (g.standard_normal(shp["b"]) * 0.02).astype(np.float32)
            elif shp:
                g = _rng(cfg.seed, 1, idx)
                std = np.sqrt(2.0 / fan_in(layer))
                p["w"] = (g.standard_normal(shp["w"]) * std).astype(np.float32)
                if bias_std > 0.0:
                    p["b"] = (g.standard_normal(shp["b"]) * bias_std).astype(np.float32)
                else:
                    p["b"] = np.zeros(shp["b"], dtype=np.float32)
            ps.append(p)
            idx += 1
        out.append(ps)
    return out


def make_batch(cfg, step, M=None):
    """One mini-batch: (x fp32 [M, *in_shape], labels int32 [M]); bf16 configs get bf16-grid inputs."""
    M = cfg.M if M is None else M
    g = _rng(cfg.seed, 2, step)
    if getattr(cfg, "vocab", 0):
        s = cfg.in_shape[0]
        t = g.integers(0, cfg.vocab, size=(M, s + 1), dtype=np.int64).astype(np.int32)
        return np.ascontiguousarray(t[:, :s]), np.ascontiguousarray(t[:, 1:])
    x = g.standard_normal((M,) + tuple(cfg.in_shape)).astype(np.float32)
    if cfg.dtype == "bf16":
        x = to_bf16_grid(x)
    y = g.integers(0, cfg.classes, size=(M,), dtype=np.int64).astype(np.int32)
    return x, y
