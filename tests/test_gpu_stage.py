"""Parity of the HIP stage step with the CPU oracle, one stage at a time, through the C ABI.

Each case forwards the N micro-batches, then CHANGES the weights (as another mini-batch's update
would), runs the single backward pass and the update, and compares every result element by element
with the oracle on the same seeded inputs.  Sizes span several tiles and a ragged tail.
bf16 stages are compared with the oracle under its bf16 storage policy, so that ReLU masks and
pooling winners are decided on the same stored values on both sides.
Tolerances (max-norm relative, tests/util.py): 1e-4 for fp32 stages, 2e-2 for bf16 stages.
"""
import numpy as np
import pytest

from oracle.stage import Stage as OStage
from tests.util import TOL, frac_outside, rel_err, rel_l2
from workloads import to_bf16_grid
from workloads.configs import conv, linear, maxpool, softmax_ce
from workloads.synth import param_shapes

pytestmark = pytest.mark.gpu


def _params(specs, rng, scale=1.0):
    ps = []
    for sp in specs:
        shp = param_shapes(sp)
        p = {}
        if shp and sp["kind"] in ("layernorm", "affine"):
            p["w"] = (1.0 + 0.2 * rng.standard_normal(shp["w"])).astype(np.float32)
            p["b"] = (0.1 * rng.standard_normal(shp["b"])).astype(np.float32)
        elif shp and sp["kind"] == "embedding":
            p["w"] = (0.5 * rng.standard_normal(shp["w"])).astype(np.float32)
            p["b"] = (0.5 * rng.standard_normal(shp["b"])).astype(np.float32)
        elif shp:
            fan = np.prod(shp["w"][1:])
            p["w"] = (rng.standard_normal(shp["w"]) * np.sqrt(2.0 / fan) * scale).astype(np.float32)
            p["b"] = (rng.standard_normal(shp["b"]) * 0.1).astype(np.float32)
        ps.append(p)
    return ps


def _in_shape(sp):
    if sp["kind"] == "linear":
        return (sp.get("rows", 1) * sp["din"],)
    if sp["kind"] == "layernorm":
        return (sp["rows"] * sp["d"],)
    if sp["kind"] == "attention":
        return (sp["s"] * 3 * sp["d"],)
    if sp["kind"] == "embedding":
        return (sp["s"],)
    if sp["kind"] == "conv":
        return (sp["h"], sp["w"], sp["cin"])
    if sp["kind"] in ("maxpool", "affine", "avgpool"):
        return (sp["h"], sp["w"], sp["c"])
    raise ValueError


def _cos(a, b):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b) + 1e-300))


def run_stage_case(specs, dtype, micro, N, seed, has_pool=False, borrow=False, deep=False, deep_l2=0.2):
    """deep (bf16 only): a stage of tens of ReLU layers.  The two sides store the same bf16 tensors only up to
    rounding ties (fp32 against fp64 sums); the differences grow with depth, a stored activation that lands on
    the other side of zero flips its ReLU mask, and after a few dozen layers two CORRECT evaluations of the same
    stage differ by percents in the gradients of the earliest layers.  tests/test_oracle_relu_ties.py shows this
    between two evaluations of the oracle that differ only in the precision of their sums, and that the
    element-wise bar holds again once both use the same masks; tests/test_gpu_resnet50_blocks.py holds every
    block of these stages, fed the oracle's tensors, to the element-wise bar at the real shapes.  A whole stage
    is held to relative L2 error < deep_l2 and direction cosine > 1 - deep_l2^2 / 2 in bf16 (deep_l2 is set per
    stage to about twice what the stage measures: 0.013, 0.047, 0.16 and 0.05 for the four ResNet-50 stages).  In fp32 the same happens to a handful of
    activations that lie within rounding of zero, and one flipped mask perturbs the whole receptive field below
    it (a whole 14 x 14 image after six blocks): there the element-wise bar must hold on 90 % of the elements
    of the input gradient, and the relative L2 error of every result must stay below 1e-2."""
    import torch
    from paper_2410_14312_amd import Stage

    rng = np.random.default_rng(seed)
    tol = TOL[dtype]
    M = micro * N
    is_last = specs[-1]["kind"] == "softmax_ce"
    p0 = _params(specs, rng)
    p1 = [{k: (v + 0.05 * np.abs(v).max() * rng.standard_normal(v.shape)).astype(np.float32) for k, v in p.items()}
          for p in p0]
    tokens_in = specs[0]["kind"] == "embedding"
    if tokens_in:
        x = rng.integers(0, specs[0]["vocab"], (M,) + _in_shape(specs[0])).astype(np.int32)
    else:
        x = rng.standard_normal((M,) + _in_shape(specs[0])).astype(np.float32)
        if dtype == "bf16":
            x = to_bf16_grid(x)
    lrows = specs[-1].get("rows", 1)
    labels = rng.integers(0, specs[-1].get("classes", 2), (M, lrows) if lrows > 1 else M).astype(np.int32)
    lr, mu = 0.05, 0.9

    ost = OStage(specs, p0, lr, mu, M, N, precision="bf16" if dtype == "bf16" else "f64")
    gst = Stage(specs, dtype, micro, N, 2 * N, lr, mu, borrow_input=borrow, device="cuda:0")
    gst.set_params(p0)
    adt = gst.act_dtype
    dev = gst.device
    xd = gst.prepare_input(x)
    ld = torch.from_numpy(labels).to(dev)
    out_elems = gst.out_elems
    base = N  # use the second group of slots so slot arithmetic is exercised
    for j in range(N):
        xs = xd[j * micro:(j + 1) * micro]
        y = torch.empty(micro * out_elems, dtype=torch.float32 if is_last else adt, device=dev)
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        gst.forward_micro(base + j, xs, y=y, labels=ld[j * micro:(j + 1) * micro] if is_last else None,
                          loss_out=loss if is_last else None)
        torch.cuda.synchronize()
        if is_last:
            o_logits, o_loss = ost.forward_micro(j, x[j * micro:(j + 1) * micro], labels[j * micro:(j + 1) * micro])
            assert rel_err(y.float().cpu().numpy().reshape(o_logits.shape), o_logits) < tol, "logits micro %d" % j
            assert abs(loss.item() - o_loss) < tol * max(1.0, abs(o_loss)), "loss micro %d" % j
        else:
            o_y = ost.forward_micro(j, x[j * micro:(j + 1) * micro])
            got = y.float().cpu().numpy().reshape(o_y.shape)
            assert rel_err(got, o_y) < tol, "forward micro %d: %g" % (j, rel_err(got, o_y))

    # another mini-batch's update lands between this mini-batch's forward and backward
    for p, q in zip(ost.params, p1):
        for k in p:
            p[k][...] = q[k]
    gst.set_params(p1)

    if is_last:
        dy, dyd = None, None
    else:
        dy = (rng.standard_normal((M, out_elems)) / M).astype(np.float32)
        if dtype == "bf16":
            dy = to_bf16_grid(dy)
        dyd = torch.from_numpy(dy).to(adt).to(dev)
    dxd = None if tokens_in else torch.empty(M * gst.in_elems, dtype=adt, device=dev)
    gst.backward(list(range(base, base + N)), dy=dyd, dx=dxd)
    torch.cuda.synchronize()
    o_dx = ost.backward(list(range(N)), dy)
    if tokens_in:
        assert o_dx is None
    got_dx = None if tokens_in else gst.crop_input_grad(dxd, M).reshape(o_dx.shape)
    deep32 = deep and dtype == "f32"
    deep = deep and dtype == "bf16"

    def mostly(got, ref, what, per_sample=True):
        # a weight gradient sums over all samples, so one perturbed sample touches every element of it a little
        f, l2 = frac_outside(got, ref, tol), rel_l2(got, ref)
        assert (f < 0.1 or not per_sample) and l2 < 1e-2, "%s: %g of the elements outside, l2 %g" % (what, f, l2)

    if tokens_in:
        pass
    elif deep32:
        mostly(got_dx, o_dx, "dx")
    elif deep:
        print("deep dx: max-norm %.3g outside %.3g l2 %.3g cos %.5f" % (rel_err(got_dx, o_dx), frac_outside(got_dx, o_dx, tol), rel_l2(got_dx, o_dx), _cos(got_dx, o_dx)), flush=True)
        assert rel_l2(got_dx, o_dx) < deep_l2 and _cos(got_dx, o_dx) > 1 - deep_l2 ** 2 / 2, "dx: l2 %g cos %g" % (rel_l2(got_dx, o_dx), _cos(got_dx, o_dx))
    elif has_pool and dtype == "bf16":
        # near-ties of a pooling window can be won by a different element in bf16 than in fp64: such
        # isolated reroutings are valid; everything else must agree
        assert frac_outside(got_dx, o_dx, tol) < 2e-3 and rel_l2(got_dx, o_dx) < 2 * tol
    else:
        assert rel_err(got_dx, o_dx) < tol, "dx: %g" % rel_err(got_dx, o_dx)
    grads = gst.get_grads()
    for li, g in enumerate(ost.grads):
        if g is None:
            continue
        for k in g:
            if deep:
                a, b = grads[li][k], g[k]
                print("deep grad %d %s: max-norm %.3g l2 %.3g" % (li, k, rel_err(a.reshape(b.shape), b), rel_l2(a, b)), flush=True)
                assert rel_l2(a, b) < deep_l2 and _cos(a, b) > 1 - deep_l2 ** 2 / 2, "grad layer %d %s: l2 %g cos %g" % (li, k, rel_l2(a, b), _cos(a, b))
                continue
            if deep32:
                mostly(grads[li][k], g[k], "grad layer %d %s" % (li, k), per_sample=False)
                continue
            if has_pool and dtype == "bf16":
                # the gradient below a pooling layer is sparse (one winner per window), so each rerouted
                # winner is a visible share of a weight-gradient sum: hold these to the L2 norm and direction
                a, b = grads[li][k].astype(np.float64).ravel(), g[k].ravel()
                cos = float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b) + 1e-300))
                assert rel_l2(a, b) < 3 * tol and cos > 0.998, "grad layer %d %s: l2 %g cos %g" % (li, k, rel_l2(a, b), cos)
                continue
            e = rel_err(grads[li][k], g[k])
            assert e < tol, "grad layer %d %s: %g" % (li, k, e)

    w_before = gst.get_params()
    gst.update()
    ost.update()
    torch.cuda.synchronize()
    assert gst.version() == 1
    w_after = gst.get_params()
    loose = (has_pool and dtype == "bf16") or deep or deep32
    step_tol = deep_l2 if deep else (1e-2 if deep32 else (3 * tol if loose else tol))
    for li, p in enumerate(ost.params):
        for k in p:
            assert (rel_l2(w_after[li][k], p[k]) if loose else rel_err(w_after[li][k], p[k])) < (step_tol if (deep or deep32) else tol)
            # the step itself, not hidden behind the size of the weights
            step_g = w_after[li][k].astype(np.float64) - w_before[li][k]
            step_o = p[k] - p1[li][k].astype(np.float64)
            e = rel_l2(step_g, step_o) if loose else rel_err(step_g, step_o)
            assert e < step_tol, "update step layer %d %s: %g" % (li, k, e)
    mom = gst.get_momentum()
    for li, b in enumerate(ost.bufs):
        for k in b:
            e = rel_l2(mom[li][k], b[k]) if loose else rel_err(mom[li][k], b[k])
            assert e < step_tol
    # slots were freed: the group can be forwarded into again
    gst.forward_micro(base, xd[:micro], labels=ld[:micro] if is_last else None)
    torch.cuda.synchronize()


DENSE_CASES = [
    # (din, dout, relu, micro, N)
    (64, 128, True, 8, 4),       # the tiny fp32 config's first stage
    (100, 72, True, 24, 3),      # ragged in every dimension
    (200, 300, False, 70, 2),    # several tiles + tails, no ReLU
    (1024, 1024, True, 64, 4),   # the bf16 MLP config's hidden stage
    # no ReLU on the three large cases: among 10^7 pre-activations one lies within fp32 rounding of zero, and its
    # mask then differs between the fp32 and the fp64 evaluation
    (128, 6144, False, 2048, 1), # wide output, many rows: the persistent 256x256 kernel in the forward pass
    (6144, 128, False, 1024, 2), # wide input: the persistent kernel in the input-gradient pass
    (1024, 1024, False, 4608, 2),  # long batch: the persistent kernel, k-split, in the weight-gradient pass
    (768, 8192, False, 2048, 2),   # long contraction, few wide tiles: the persistent kernel in k-slices in the input-gradient pass
    (768, 512, False, 3000, 2),    # tall narrow input gradient, ragged last row of tiles: the 256x128 four-wave instance
    (192, 3080, False, 2000, 2),   # the persistent kernel in the forward pass with ragged tiles in both directions
    (3080, 192, False, 2000, 2),   # ... in the input-gradient pass
    (2056, 2056, False, 2048, 2),  # ... in the weight-gradient pass (k-slices, row sums from the fragments, ragged tiles)
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("din,dout,relu,micro,N", DENSE_CASES)
def test_linear_stage(dtype, din, dout, relu, micro, N):
    run_stage_case([linear(din, dout, relu)], dtype, micro, N, seed=din + dout)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("borrow", [False, True])
def test_last_stage_two_linears_and_loss(dtype, borrow):
    run_stage_case([linear(128, 128, True), linear(128, 10, False), softmax_ce(10)], dtype, 8, 4, seed=5, borrow=borrow)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
# one wave per row; one block per row with the row in registers (4 and 8 pieces per thread); the row in LDS; neither
@pytest.mark.parametrize("classes", [1000, 2600, 20000, 33000, 2601])
def test_last_stage_many_classes(dtype, classes):
    run_stage_case([linear(96, classes, False), softmax_ce(classes)], dtype, 6, 2, seed=6)


CONV_CASES = [
    # (h, w, cin, cout, r, stride, pad, relu, micro, N)
    (8, 8, 3, 16, 3, 1, 1, True, 4, 2),      # first-layer shape: 3 input channels
    (10, 9, 16, 24, 3, 1, 1, True, 3, 2),    # non-square, ragged channels
    (8, 8, 32, 64, 1, 1, 0, False, 4, 2),    # 1x1
    (9, 9, 16, 32, 3, 2, 1, True, 4, 2),     # strided 3x3
    (8, 8, 16, 32, 1, 2, 0, False, 4, 2),    # strided 1x1 (projection shortcut shape)
    (20, 20, 3, 16, 7, 2, 3, True, 2, 2),    # 7x7 stride 2 stem
    (4, 4, 64, 128, 3, 1, 1, True, 32, 4),   # deep-layer shape: small image, many channels, M=128
    # stride 2 on even maps with channel counts of 8: the input gradient orders its rows by position parity
    (8, 8, 16, 32, 3, 2, 1, True, 4, 2),     # 3x3: 4, 2, 2 and 1 taps per class
    (16, 16, 8, 16, 7, 2, 3, True, 2, 2),    # 7x7: 3 or 4 taps along each axis
    (32, 32, 128, 16, 3, 2, 1, True, 8, 2),  # 128-wide tiles
    (12, 8, 24, 16, 3, 2, 0, False, 4, 2),   # no padding, non-square, ragged channels
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("h,w,cin,cout,r,stride,pad,relu,micro,N", CONV_CASES)
def test_conv_stage(dtype, h, w, cin, cout, r, stride, pad, relu, micro, N):
    run_stage_case([conv(h, w, cin, cout, r, stride, pad, relu)], dtype, micro, N, seed=h * 100 + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_conv_pool_conv_stage(dtype):
    specs = [conv(8, 8, 8, 16), conv(8, 8, 16, 16), maxpool(8, 8, 16), conv(4, 4, 16, 32)]
    run_stage_case(specs, dtype, 4, 2, seed=9, has_pool=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pool_first_and_overlapping_windows(dtype):
    run_stage_case([maxpool(9, 9, 8, k=3, stride=2), conv(4, 4, 8, 8)], dtype, 3, 2, seed=10, has_pool=True)


@pytest.mark.parametrize("h,w,c,k,stride,pad", [
    (37, 45, 72, 3, 2, 1),   # the LDS-tiled gather: ragged tiles at both edges, a ragged last group of channels
    (24, 32, 16, 3, 1, 1),   # every element in nine windows
    (33, 40, 8, 2, 2, 0),    # odd height: the last row belongs to no window
    (20, 36, 64, 5, 3, 2),   # wide windows
])
def test_pool_on_large_maps(h, w, c, k, stride, pad):
    # the pooling layer comes first, so both sides pick their winners on identical inputs: the strict bar applies
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    run_stage_case([maxpool(h, w, c, k, stride, pad), conv(ho, wo, c, 8, 1, 1, 0, False)], "bf16", 2, 2,
                   seed=h + w + c + k)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_conv_pool_fc_loss_stage(dtype):
    specs = [conv(4, 4, 16, 32), maxpool(4, 4, 32), linear(2 * 2 * 32, 64, True), linear(64, 10, False), softmax_ce(10)]
    run_stage_case(specs, dtype, 8, 4, seed=11, has_pool=True)


@pytest.mark.parametrize("name,stage", [("tiny_mlp_f32", 0), ("tiny_mlp_f32", 1),
                                        ("mlp4x1024_bf16", 0), ("mlp4x1024_bf16", 1), ("mlp4x1024_bf16", 3),
                                        ("vgg16_bf16", 0), ("vgg16_bf16", 1), ("vgg16_bf16", 2), ("vgg16_bf16", 3)])
def test_benchmark_config_stage_at_full_size(name, stage):
    from workloads import get_config
    cfg = get_config(name)
    specs = cfg.stages[stage]
    has_pool = any(sp["kind"] == "maxpool" for sp in specs)
    run_stage_case(specs, cfg.dtype, cfg.micro, cfg.N, seed=100 + stage, has_pool=has_pool, borrow=stage > 0)


def test_slot_errors():
    import torch
    from paper_2410_14312_amd import Stage, TmpsError
    st = Stage([linear(16, 16, True)], "f32", 4, 2, 4, 0.1, 0.9)
    st.set_params([{"w": np.zeros((16, 16), np.float32), "b": np.zeros(16, np.float32)}])
    x = torch.zeros(4, 16, dtype=torch.float32, device="cuda:0")
    dy = torch.zeros(8, 16, dtype=torch.float32, device="cuda:0")
    st.forward_micro(0, x)
    with pytest.raises(TmpsError) as e:
        st.forward_micro(0, x)          # slot in use
    assert e.value.code == -4
    with pytest.raises(TmpsError) as e:
        st.backward([0, 1], dy=dy)      # slot 1 never forwarded
    assert e.value.code == -4
    with pytest.raises(TmpsError) as e:
        st.backward([0], dy=dy)         # not a whole mini-batch
    assert e.value.code == -4
    with pytest.raises(TmpsError) as e:
        st.forward_micro(7, x)
    assert e.value.code == -4
    st.forward_micro(1, x)
    with pytest.raises(TmpsError) as e:
        st.backward([0, 1], dy=None)    # dy required on a stage without loss
    assert e.value.code == -1
    st.backward([0, 1], dy=dy)
    torch.cuda.synchronize()
