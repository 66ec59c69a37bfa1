"""tmps_forward_micro_static (the forward pass with its contraction workspace in a fixed array of the library's
device code, for callers that cannot allocate) against tmps_forward_micro, through the C ABI.

The kernels are the same and take the workspace as an argument, so the results must agree bit for bit (which is
inside the bar of every dtype).  Two calls in a row, the second on a smaller stage, so that the second call runs on
a workspace that still holds the first call's partial sums; the shapes are chosen so that the contractions ARE
split along k (few output tiles, long contraction) and the workspace is really used.
"""
import numpy as np
import pytest

from workloads import to_bf16_grid
from workloads.configs import conv, linear, softmax_ce

pytestmark = pytest.mark.gpu


def _stage(specs, dtype, micro, seed):
    from paper_2410_14312_amd import Stage
    from tests.test_gpu_stage import _params
    rng = np.random.default_rng(seed)
    st = Stage(specs, dtype, micro, 2, 2, 0.05, 0.9, device="cuda:0")
    st.set_params(_params(specs, rng))
    return st, rng


def _both_ways(specs, dtype, micro, seed, in_shape, classes=0):
    import torch
    st, rng = _stage(specs, dtype, micro, seed)
    x = rng.standard_normal((micro,) + in_shape).astype(np.float32)
    xd = st.prepare_input(to_bf16_grid(x) if dtype == "bf16" else x)
    last = classes > 0
    lab = torch.from_numpy(rng.integers(0, max(classes, 1), micro).astype(np.int32)).to(st.device) if last else None
    outs = []
    for slot, call in ((0, st.forward_micro), (1, st.forward_micro_static)):
        y = torch.full((micro * st.out_elems,), float("nan"), dtype=torch.float32 if last else st.act_dtype, device=st.device)
        loss = torch.full((1,), float("nan"), dtype=torch.float32, device=st.device)
        call(slot, xd, y=y, labels=lab, loss_out=loss if last else None)
        torch.cuda.synchronize()
        outs.append((y.float().cpu().numpy(), loss.item()))
    (ya, la), (yb, lb) = outs
    assert np.isfinite(ya).all()
    assert np.array_equal(ya, yb), "static-workspace forward differs from tmps_forward_micro"
    if last:
        assert la == lb and np.isfinite(la)
    return st


def test_static_workspace_forward_twice_second_call_smaller():
    # 64 x 1024 outputs from a contraction of 3072: 16 tiles, split along k; then a classifier with a ragged logits layer
    big = _both_ways([linear(3072, 1024, True), linear(1024, 1024, True)], "bf16", 64, 1, (3072,))
    assert big is not None
    small = _both_ways([conv(4, 4, 64, 128, 3, 1, 1, True), linear(4 * 4 * 128, 10, False), softmax_ce(10)], "bf16", 16, 2,
                       (4, 4, 64), classes=10)
    assert small is not None
    # fp32 stages take the same entry point
    _both_ways([linear(1536, 96, True)], "f32", 24, 3, (1536,))


def test_static_workspace_rejects_a_stage_that_needs_more():
    import torch
    from paper_2410_14312_amd import Stage, TmpsError
    # 1536 x 2048 outputs over a contraction of 8192: two k-slices of fp32 partial tiles are 37.7 MB, the array holds 32 MiB
    st = Stage([linear(8192, 2048, False)], "bf16", 1536, 1, 1, 0.05, 0.9, device="cuda:0")
    x = torch.zeros(1536, 8192, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(TmpsError) as e:
        st.forward_micro_static(0, x)
    assert e.value.code == -8 and "workspace" in str(e.value)
    st.forward_micro(0, x)      # the slot is still free: nothing was launched, and the ordinary call takes it
    torch.cuda.synchronize()
