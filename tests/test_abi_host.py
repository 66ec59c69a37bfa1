"""Host-side checks of the C ABI: every declared symbol is exported, the schedule planner agrees
bit for bit with the oracle's simulation, and layout/argument errors are reported, not crashed on.
No GPU is touched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2410_14312_amd as T
from paper_2410_14312_amd import binding as B
from oracle import schedule as S
from workloads.configs import conv, linear, maxpool, softmax_ce

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported_and_bound():
    text = open(os.path.join(ROOT, "include", "tmps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(tmps_[a-z_0-9]+)\s*\(", text))
    assert len(declared) >= 19
    lib = T.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)


@pytest.mark.parametrize("W,N,n", [(1, 4, 3), (2, 4, 20), (4, 4, 9), (4, 2, 9), (4, 8, 6), (3, 2, 7),
                                   (5, 2, 12), (5, 3, 12), (8, 3, 20), (6, 2, 15), (2, 1, 4), (3, 1, 5)])
def test_planner_equals_oracle_simulation(W, N, n):
    got = T.schedule_plan(W, N, n)
    want = np.array(S.simulate(W, N, n)["ops"], dtype=np.int32)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


@pytest.mark.parametrize("W,n", [(1, 5), (2, 9), (3, 7), (4, 12), (7, 30)])
def test_1f1b_planner_equals_oracle_simulation(W, n):
    from oracle import baseline
    got = T.schedule_plan_1f1b(W, n)
    want = np.array(baseline.simulate_1f1b(W, n), dtype=np.int32)
    assert got.shape == want.shape and np.array_equal(got, want)
    with pytest.raises(T.TmpsError):
        T.schedule_plan_1f1b(0, 3)


def test_version_difference_exports():
    for W in range(2, 11):
        for N in range(2, 8):
            assert T.version_diff_formula(W, N) == (W + N - 2) // N
            assert T.version_diff_simulated(W, N) == S.version_difference_simulated(W, N)
            need = S.stash_groups_needed(W, N, 3 * W + 4)
            for s in range(W):
                assert T.schedule_stash_groups(W, N, s) == need[s]
    with pytest.raises(T.TmpsError) as e:
        T.version_diff_formula(1, 4)
    assert e.value.code == -1


def test_plan_capacity_error():
    buf = (C.c_int32 * 7)()
    rc = T.lib().tmps_schedule_plan(4, 4, 3, buf, 1)
    assert rc == -8 and b"needed" in T.lib().tmps_last_error()


def _cfg(dtype=0, micro=8, N=4, stash=4, last=0, borrow=0):
    return B.StageCfg(dtype, micro, N, stash, last, borrow, 0.01, 0.9)


def test_stage_bytes_layout_and_errors():
    specs = [linear(64, 128, True)]
    p, s, st, sc = B.stage_bytes(specs, _cfg())
    P = 64 * 128 + 128
    assert p >= P * 4 and s >= P * 8 and st >= 4 * 8 * (64 + 128) * 4 and sc > 0
    p16, _, st16, _ = B.stage_bytes(specs, _cfg(dtype=1))
    assert p16 >= P * 6 and st16 < st
    # unequal micro-batches: stash capacity not a whole number of mini-batches
    with pytest.raises(T.TmpsError) as e:
        B.stage_bytes(specs, _cfg(stash=6))
    assert e.value.code == -3
    # layers that do not chain
    with pytest.raises(T.TmpsError) as e:
        B.stage_bytes([linear(64, 128, True), linear(100, 10, False)], _cfg())
    assert e.value.code == -2
    # loss anywhere but at the end of the last stage
    with pytest.raises(T.TmpsError) as e:
        B.stage_bytes([linear(64, 10, False), softmax_ce(10)], _cfg(last=0))
    assert e.value.code == -2
    with pytest.raises(T.TmpsError) as e:
        B.stage_bytes([linear(64, 10, False)], _cfg(last=1))
    assert e.value.code == -2
    # conv -> pool -> linear chain is accepted
    ok = [conv(8, 8, 3, 16), maxpool(8, 8, 16), linear(4 * 4 * 16, 10, False), softmax_ce(10)]
    assert all(v > 0 for v in B.stage_bytes(ok, _cfg(last=1)))
    with pytest.raises(T.TmpsError):
        B.stage_bytes([conv(8, 8, 3, 16), linear(100, 10, False)], _cfg())


def test_create_rejects_null_and_misaligned_regions():
    descs = B.layer_descs([linear(8, 8, False)])
    cfg = _cfg()
    h = C.c_void_p()
    rc = T.lib().tmps_stage_create(C.byref(h), descs, 1, C.byref(cfg), None, None, None, None)
    assert rc == -1 and h.value is None
    rc = T.lib().tmps_stage_create(C.byref(h), descs, 1, C.byref(cfg), 0x1001, 0x1000, 0x1000, 0x1000)
    assert rc == -1 and h.value is None
