"""Graph replay (tmps_stage_use_graphs) against the kernel-by-kernel path of the same library: the same kernels in the
same order, so every result must be equal bit for bit, on the first call with a set of addresses (which runs directly),
on the second (which is captured, instantiated and launched) and on every replay after it, with the program's own
synchronisations and host reads between the replays.  The kernel-by-kernel path itself is held to the CPU oracle by the
other GPU tests.
"""
import numpy as np
import pytest

from workloads import get_config, init_params, make_batch
from workloads.configs import linear, softmax_ce, transformer_block, layernorm

pytestmark = pytest.mark.gpu


def _stage_pair(specs, dtype, micro, N, last):
    import torch
    from paper_2410_14312_amd import Stage
    from tests.test_gpu_stage import _params
    rng = np.random.default_rng(3)
    params = _params(specs, rng)
    pair = []
    for graphs in (False, True):
        st = Stage(specs, dtype, micro, N, 2 * N, 1e-3, 0.9, borrow_input=False, device="cuda:0")
        st.set_params(params)
        if graphs:
            st.use_graphs(True)
        pair.append(st)
    return pair


def _same(a, b, what):
    import torch
    assert bool(torch.isfinite(a.float()).all()), what + ": not finite"
    assert torch.equal(a, b), what


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["mlp", "mlp_last", "transformer", "transformer_last"])
def test_stage_passes_replayed_from_graphs(dtype, kind):
    import torch
    micro, N = 4, 2
    if kind.startswith("mlp"):
        din, rows, classes = 64, 1, 24
        specs = [linear(din, 96, True), linear(96, 48, True)]
        if kind.endswith("last"):
            specs += [linear(48, classes, False), softmax_ce(classes)]
    else:
        s_len, d, classes = 24, 64, 40
        din, rows = s_len * d, s_len
        specs = transformer_block(s_len, d, 2, 128)
        if kind.endswith("last"):
            specs += [layernorm(d, s_len), linear(d, classes, False, rows=s_len), softmax_ce(classes, rows=s_len)]
    last = kind.endswith("last")
    eager, graph = _stage_pair(specs, dtype, micro, N, last)
    adt = eager.act_dtype
    gen = torch.Generator(device="cuda").manual_seed(5)
    M = micro * N
    stream = torch.cuda.Stream()   # (the default stream cannot be captured: passes issued there always run directly)
    for step in range(5):
        # new values at the same addresses every step: the second step is the captured one, later ones replay
        if step == 0:
            x = torch.empty(M, din, device="cuda", dtype=adt)
            dy = None
            labels = torch.empty(M, rows, device="cuda", dtype=torch.int32) if last else None
            dx = [torch.empty(M, din, device="cuda", dtype=adt) for _ in range(2)]
            loss = [torch.zeros(N, device="cuda", dtype=torch.float32) for _ in range(2)]
        x.copy_(torch.randn(M, din, device="cuda", generator=gen).to(adt))
        if last:
            labels.copy_(torch.randint(0, classes, (M, rows), device="cuda", generator=gen, dtype=torch.int32))
        if not last:
            if dy is None:
                dy = torch.empty(M, eager.out_elems, device="cuda", dtype=adt)
            dy.copy_(torch.randn(M, eager.out_elems, device="cuda", generator=gen).to(adt))
        torch.cuda.synchronize()
        outs = []
        for k, st in enumerate((eager, graph)):
            ys = []
            for j in range(N):
                y = None if last else torch.empty(micro, st.out_elems, device="cuda", dtype=adt)
                st.forward_micro(j, x[j * micro:(j + 1) * micro],
                                 y=y, labels=labels[j * micro:(j + 1) * micro] if last else None,
                                 loss_out=loss[k][j:j + 1] if last else None, stream=stream)
                ys.append(y)
            outs.append(ys)
        torch.cuda.synchronize()
        if not last:
            for j in range(N):
                _same(outs[0][j], outs[1][j], "step %d: output of micro-batch %d" % (step, j))
        else:
            _same(loss[0], loss[1], "step %d: losses" % step)
        for k, st in enumerate((eager, graph)):
            st.backward(list(range(N)), dy=dy, dx=dx[k], stream=stream)
            st.update(stream=stream)
        torch.cuda.synchronize()
        _same(dx[0], dx[1], "step %d: input gradient" % step)
        ge, gg = eager.get_grads(), graph.get_grads()
        pe, pg = eager.get_params(), graph.get_params()
        for li in range(len(pe)):
            for name in pe[li]:
                assert np.array_equal(ge[li][name], gg[li][name]), "step %d: gradient of layer %d %s" % (step, li, name)
                assert np.array_equal(pe[li][name], pg[li][name]), "step %d: layer %d %s" % (step, li, name)
    assert eager.version() == graph.version() == 5


@pytest.mark.parametrize("name,steps", [("tiny_mlp_f32", 8), ("tiny_transformer_bf16", 6), ("tiny_resnet_bf16", 6),
                                        ("mlp4x1024_bf16", 6)])
def test_pipeline_run_replayed_from_graphs(name, steps):
    # the emulator's K-stream run, with host threads issuing: every loss, every parameter and the version log of a run
    # that replays graphs equal those of the kernel-by-kernel run; a second run on the same stages (all graphs exist by
    # then) continues to agree
    from paper_2410_14312_amd import Pipeline
    cfg = get_config(name)
    params = init_params(cfg)
    pipes = [Pipeline(cfg, params), Pipeline(cfg, params, graphs=True)]
    for rnd in range(2):
        batches = [make_batch(cfg, rnd * steps + i) for i in range(steps)]
        res = [p.run(batches) for p in pipes]
        assert res[0][0] == res[1][0], "losses of run %d" % rnd
        assert np.array_equal(res[0][1], res[1][1]), "version log of run %d" % rnd
        for s in range(cfg.K):
            a, b = pipes[0].get_params(s), pipes[1].get_params(s)
            for li in range(len(a)):
                for k in a[li]:
                    assert np.array_equal(a[li][k], b[li][k]), "run %d stage %d layer %d %s" % (rnd, s, li, k)


def test_timing_switches_replay_off():
    # while per-kernel timing is on nothing is captured or replayed, and results do not change
    import torch
    from paper_2410_14312_amd import binding as B
    micro, N = 4, 2
    specs = [linear(32, 32, True), linear(32, 16, False)]
    eager, graph = _stage_pair(specs, "bf16", micro, N, False)
    x = torch.randn(micro * N, 32, device="cuda").to(eager.act_dtype)
    dy = torch.randn(micro * N, 16, device="cuda").to(eager.act_dtype)
    dx = [torch.empty(micro * N, 32, device="cuda", dtype=eager.act_dtype) for _ in range(2)]
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    for step in range(6):
        B.profile_enable(step in (3, 4))
        for k, st in enumerate((eager, graph)):
            for j in range(N):
                st.forward_micro(j, x[j * micro:(j + 1) * micro], stream=stream)
            st.backward(list(range(N)), dy=dy, dx=dx[k], stream=stream)
            st.update(stream=stream)
        torch.cuda.synchronize()
        assert torch.equal(dx[0], dx[1])
    pr = B.profile_read()
    B.profile_enable(False)
    assert pr["dense_fwd"][1] > 0   # the timed steps launched kernel by kernel, on both stages
