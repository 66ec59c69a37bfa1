"""Shape tables of the benchmark networks, as neutral layer lists.

A network is a list of stages (the paper's workers: consecutive layers on one
accelerator, Methodology / Model Architecture); a stage is a list of layer
dicts.  Per-sample activation layout is channels-last (``[H, W, C]``) or a
flat vector ``[D]``.  Nothing here computes anything: the dicts are read by
the oracle-side tests and by the HIP binding alike.
"""
from dataclasses import dataclass, field
from typing import List, Tuple


def linear(din, dout, relu, act=None, rows=1, skip=0):
    """rows: rows per sample (the layer acts on each row of [rows, din]); act: None or "gelu" (relu=True is
    the ReLU); skip: k > 0 adds the input of the layer k positions before this one (residual connection)."""
    return {"kind": "linear", "din": int(din), "dout": int(dout), "relu": bool(relu), "act": act,
            "rows": int(rows), "skip": int(skip)}


def layernorm(d, rows=1, eps=1e-5):
    return {"kind": "layernorm", "d": int(d), "rows": int(rows), "eps": float(eps)}


def attention(s, d, heads):
    """Causal multi-head self-attention on packed [s, 3d] = (q | k | v) rows; output [s, d]."""
    return {"kind": "attention", "s": int(s), "d": int(d), "heads": int(heads)}


def embedding(vocab, s, d):
    """Token + learned positional embedding: int tokens [s] -> [s, d]."""
    return {"kind": "embedding", "vocab": int(vocab), "s": int(s), "d": int(d)}


def transformer_block(s, d, heads, ffn):
    """Pre-LayerNorm block: x + proj(attn(qkv(LN(x)))), then x + fc2(gelu(fc1(LN(x))))."""
    return [layernorm(d, s), linear(d, 3 * d, False, rows=s), attention(s, d, heads),
            linear(d, d, False, rows=s, skip=3),
            layernorm(d, s), linear(d, ffn, False, act="gelu", rows=s), linear(ffn, d, False, rows=s, skip=2)]


def conv(h, w, cin, cout, r=3, stride=1, pad=1, relu=True, src=1):
    """src: which earlier result the layer reads: 1 = the layer before it (the default), k = the layer k
    positions before it; one position before the first layer of a stage is the stage input."""
    return {"kind": "conv", "h": int(h), "w": int(w), "cin": int(cin), "cout": int(cout),
            "r": int(r), "s": int(r), "stride": int(stride), "pad": int(pad), "relu": bool(relu), "src": int(src)}


def maxpool(h, w, c, k=2, stride=2, pad=0):
    """pad: rows / columns of padding on every side; padded positions never win."""
    return {"kind": "maxpool", "h": int(h), "w": int(w), "c": int(c), "k": int(k),
            "stride": int(stride), "pad": int(pad)}


def affine(h, w, c, relu, init_gain=1.0):
    """Trainable per-channel scale and shift (a batch-normalisation layer with its statistics folded away):
    y = gain[c] * x + shift[c], then ReLU if asked.  init_gain: the value the gains start from."""
    return {"kind": "affine", "h": int(h), "w": int(w), "c": int(c), "relu": bool(relu), "init_gain": float(init_gain)}


def resadd(h, w, c, src_b, relu=True):
    """y = act(a + b): a is the result of the layer before, b that of the layer src_b positions before
    (same convention as conv's src): the join of a residual connection."""
    return {"kind": "resadd", "h": int(h), "w": int(w), "c": int(c), "src_b": int(src_b), "relu": bool(relu)}


def avgpool(h, w, c):
    """Mean over all h*w positions: [h, w, c] -> [c]."""
    return {"kind": "avgpool", "h": int(h), "w": int(w), "c": int(c)}


def bottleneck(h, cin, width, stride, project):
    """ResNet bottleneck block on an h x h x cin input: 1x1 (width) - 3x3 (width, stride) - 1x1 (4 width), each
    followed by a per-channel affine layer, ReLU after the first two; the block input (or, in the first block
    of a group, a strided 1x1 projection of it with its own affine layer) is added before the last ReLU.
    The last affine layer of the main path starts from gain 0.2: with no batch statistics to renormalise them,
    sixteen blocks that each add a full-size branch to their input would grow the activations and gradients
    by orders of magnitude, and plain SGD at the configured rate diverges within a few steps."""
    ho = (h + 2 - 3) // stride + 1
    cout = 4 * width
    layers = [conv(h, h, cin, width, 1, 1, 0, False), affine(h, h, width, True),
              conv(h, h, width, width, 3, stride, 1, False), affine(ho, ho, width, True),
              conv(ho, ho, width, cout, 1, 1, 0, False), affine(ho, ho, cout, False, init_gain=0.2)]
    if project:
        # the projection reads the block input: 7 positions before itself
        layers += [conv(h, h, cin, cout, 1, stride, 0, False, src=7), affine(ho, ho, cout, False),
                   resadd(ho, ho, cout, src_b=1 + 2, relu=True)]
        # resadd: a = the projection's affine (the layer before), b = the main path's affine, 3 positions before
    else:
        layers += [resadd(ho, ho, cout, src_b=7, relu=True)]   # b = the block input
    return layers, ho, cout


def softmax_ce(classes, rows=1):
    """rows: labelled rows per sample (sequence positions); the loss is the mean over all rows."""
    return {"kind": "softmax_ce", "classes": int(classes), "rows": int(rows)}


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
    vocab: int = 0             # > 0: inputs are int token ids [S] uniform over the vocabulary, labels the next tokens

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


def _transformer(name, dtype, layers, d, heads, ffn, s, vocab, M, N, K, seed):
    per = layers // K
    stages = []
    for k in range(K):
        st = [embedding(vocab, s, d)] if k == 0 else []
        for _ in range(per):
            st += transformer_block(s, d, heads, ffn)
        if k == K - 1:
            st += [layernorm(d, s), linear(d, vocab, False, rows=s), softmax_ce(vocab, rows=s)]
        stages.append(st)
    return Config(name=name, dtype=dtype, M=M, N=N, seed=seed, steps=2, in_shape=(s,), classes=vocab, vocab=vocab,
                  stages=stages,
                  notes="pre-LayerNorm, causal attention, exact-erf GELU, learned positions, untied output layer, "
                        "eps 1e-5; S+1 tokens are drawn per sample: the first S are the input, the last S the targets")


def _resnet(name, dtype, size, widths, blocks, classes, M, N, seed, stem_c=64):
    """Bottleneck residual network on size x size x 3 images, one stage per group of blocks (the stem joins the
    first group, the classifier the last)."""
    h = (size + 2 * 3 - 7) // 2 + 1
    stem = [conv(size, size, 3, stem_c, 7, 2, 3, False), affine(h, h, stem_c, True), maxpool(h, h, stem_c, 3, 2, 1)]
    h = (h + 2 - 3) // 2 + 1
    cin = stem_c
    stages = []
    for gi, (w, nb) in enumerate(zip(widths, blocks)):
        st = stem if gi == 0 else []
        for bi in range(nb):
            ls, h, cin = bottleneck(h, cin, w, 2 if (bi == 0 and gi > 0) else 1, bi == 0)
            st = st + ls
        if gi == len(widths) - 1:
            st = st + [avgpool(h, h, cin), linear(cin, classes, False), softmax_ce(classes)]
        stages.append(st)
    return Config(name=name, dtype=dtype, M=M, N=N, seed=seed, steps=2, in_shape=(size, size, 3), classes=classes,
                  stages=stages,
                  notes="bottleneck blocks, batch normalisation folded to a trainable per-channel affine layer (gain 1, "
                        "shift 0 at the start, gain 0.2 on the last affine layer of every block), stride on the 3x3, projection shortcut in the first block of each group, "
                        "bias on every convolution")


def _resnet50():
    return _resnet("resnet50_bf16", "bf16", 224, (64, 128, 256, 512), (3, 4, 6, 3), 1000, M=64, N=8, seed=3)


def _tiny_resnet(dtype):
    return lambda: _resnet("tiny_resnet_" + dtype, dtype, 32, (8, 16), (2, 2), 10, M=8, N=4, seed=6, stem_c=8)


def _gpt2_small():
    return _transformer("gpt2_small_bf16", "bf16", 12, 768, 12, 3072, 512, 32000, M=16, N=8, K=4, seed=4)


def _tiny_transformer(dtype):
    return lambda: _transformer("tiny_transformer_" + dtype, dtype, 2, 64, 2, 128, 32, 96, M=8, N=4, K=2, seed=5)


CONFIGS = {
    "tiny_mlp_f32": _tiny_mlp,
    "mlp4x1024_bf16": _mlp_bf16,
    "vgg16_bf16": _vgg16,
    "resnet50_bf16": _resnet50,
    "gpt2_small_bf16": _gpt2_small,
    "tiny_resnet_f32": _tiny_resnet("f32"),
    "tiny_resnet_bf16": _tiny_resnet("bf16"),
    "tiny_transformer_f32": _tiny_transformer("f32"),
    "tiny_transformer_bf16": _tiny_transformer("bf16"),
}


def get_config(name: str) -> Config:
    return CONFIGS[name]()


def layer_out_shape(layer, in_shape):
    """Per-sample output shape of one layer given its per-sample input shape."""
    k = layer["kind"]
    if k == "linear":
        return (layer["dout"],) if layer.get("rows", 1) == 1 else (layer["rows"], layer["dout"])
    if k == "layernorm":
        return tuple(in_shape)
    if k == "attention":
        return (layer["s"], layer["d"])
    if k == "embedding":
        return (layer["s"], layer["d"])
    if k == "conv":
        ho = (layer["h"] + 2 * layer["pad"] - layer["r"]) // layer["stride"] + 1
        wo = (layer["w"] + 2 * layer["pad"] - layer["s"]) // layer["stride"] + 1
        return (ho, wo, layer["cout"])
    if k == "maxpool":
        ho = (layer["h"] + 2 * layer.get("pad", 0) - layer["k"]) // layer["stride"] + 1
        wo = (layer["w"] + 2 * layer.get("pad", 0) - layer["k"]) // layer["stride"] + 1
        return (ho, wo, layer["c"])
    if k in ("affine", "resadd"):
        return (layer["h"], layer["w"], layer["c"])
    if k == "avgpool":
        return (layer["c"],)
    if k == "softmax_ce":
        return (layer["classes"],) if layer.get("rows", 1) == 1 else (layer["rows"], layer["classes"])
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
