"""Pins of the oracle's nF1B simulation against what the paper states about its figures."""
import os

import pytest

from oracle import schedule as S


def _read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


PAIRS = [(W, N) for W in range(2, 11) for N in range(2, 9)]


@pytest.mark.parametrize("W,N", PAIRS)
def test_forward_and_backward_durations(W, N):
    # f1 = W+N-1, f2 = f1+1, b = W  (section "Mathematical Relationship between W and N")
    sim = S.simulate(W, N, 3)
    f = {b: sim["fwd_end"][b] - sim["fwd_start"][b] + 1 for b in (1, 2)}
    assert f[1] == W + N - 1
    assert f[2] == f[1] + 1
    for b in (1, 2, 3):
        assert sim["bwd_end"][b] - sim["bwd_start"][b] + 1 == W


@pytest.mark.parametrize("W,N", PAIRS)
def test_backward_starts_right_after_forward_and_recurs_every_N_plus_1(W, N):
    sim = S.simulate(W, N, 6)
    for b in range(1, 7):
        assert sim["bwd_start"][b] == sim["fwd_end"][b] + 1
    last_stage_bwd = [op[0] for op in sim["ops"] if op[2] == S.BWD and op[1] == W - 1]
    assert all(b - a == N + 1 for a, b in zip(last_stage_bwd, last_stage_bwd[1:]))


def test_every_third_and_fifth_time_point_with_four_workers():
    # section "Work Scheduling": with W=4 backward passes come at each third (N=2) and fifth (N=4)
    # time-point after the first one, on every worker.
    for N, period in ((2, 3), (4, 5)):
        sim = S.simulate(4, N, 8)
        for s in range(4):
            ts = [op[0] for op in sim["ops"] if op[2] == S.BWD and op[1] == s]
            assert all(b - a == period for a, b in zip(ts, ts[1:]))


@pytest.mark.parametrize("W,N", PAIRS)
def test_worker_chain_is_n_forwards_then_one_backward(W, N):
    # once the first backward pass has been done, each worker repeats "N forward, 1 backward"
    sim = S.simulate(W, N, 3 * W + 6)
    for s in range(W):
        kinds = [op[2] for op in sim["ops"] if op[1] == s]
        first_b = kinds.index(S.BWD)
        tail = kinds[first_b:]
        n_full = (len(tail) - 1) // (N + 1)
        for c in range(n_full - W):           # the drain at the very end has no forwards left
            chunk = tail[1 + c * (N + 1): 1 + (c + 1) * (N + 1)]
            assert chunk == [S.FWD] * N + [S.BWD]


def test_micro_batch_1A_on_worker_2_while_1B_on_worker_1():
    # section "Overlapping of Computation and Communication"
    sim = S.simulate(4, 2, 2)
    at = {(op[3], op[4], op[1]): op[0] for op in sim["ops"] if op[2] == S.FWD}
    assert at[(1, 0, 1)] == at[(1, 1, 0)]


def test_drawn_cases_version_difference(golden_dir):
    for W, N, v in _read_table(os.path.join(golden_dir, "paper_version_difference_cases.txt")):
        W, N, v = int(W), int(N), int(v)
        assert S.version_difference_simulated(W, N) == v
        assert S.version_difference_formula(W, N) == v


def test_weight_usage_facts(golden_dir):
    for W, N, kind, b, j, seen in _read_table(os.path.join(golden_dir, "paper_weight_usage_facts.txt")):
        W, N, b, seen = int(W), int(N), int(b), int(seen)
        sim = S.simulate(W, N, b + 2)
        if kind == "B":
            got = {op[6] for op in sim["ops"] if op[2] == S.BWD and op[3] == b}
        else:
            jj = ord(j) - ord("A")
            got = {op[6] for op in sim["ops"] if op[2] == S.FWD and op[3] == b and op[4] == jj}
        assert got == {seen}, (W, N, kind, b, j, got)


def test_update_sequences():
    # section "Multiple Sequence Problem"
    assert S.update_chains(4, 2, 8) == [[1, 3, 5, 7], [2, 4, 6, 8]]
    assert S.update_chains(4, 4, 8) == [[1, 2, 3, 4, 5, 6, 7, 8]]


@pytest.mark.parametrize("W,N", PAIRS)
def test_v_is_one_iff_W_le_N_plus_1(W, N):
    assert (S.version_difference_simulated(W, N) == 1) == (W <= N + 1)
    assert (S.version_difference_formula(W, N) == 1) == (W <= N + 1)


@pytest.mark.parametrize("W,N", PAIRS)
def test_closed_form_equals_simulation_where_the_paper_derives_it(W, N):
    # The closed form is reached through the assumption x ~ 1/N and checked by the authors on
    # figures with W <= 2N+1; brute force agrees with it exactly on that region.
    if W <= 2 * N + 1:
        assert S.version_difference_formula(W, N) == S.version_difference_simulated(W, N)
    else:
        assert S.version_difference_simulated(W, N) <= S.version_difference_formula(W, N)


@pytest.mark.parametrize("W,N", PAIRS)
def test_minibatches_entered_during_first_forward(W, N):
    sim = S.simulate(W, N, W + 3)
    end1 = sim["fwd_end"][1]
    last_inject = {}
    for op in sim["ops"]:
        if op[2] == S.FWD and op[1] == 0 and op[4] == N - 1:
            last_inject[op[3]] = op[0]
    entered = sum(1 for b, t in last_inject.items() if t <= end1)
    assert entered == S.minibatches_entered_during_first_forward(W, N) == (W + N - 1) // N


@pytest.mark.parametrize("W,N", [(2, 4), (4, 4), (4, 8), (3, 2), (5, 4)])
def test_at_v1_every_backward_reads_stage_version_b_minus_1(W, N):
    sim = S.simulate(W, N, 9)
    for (t, s, kind, b, j, sv, nv) in sim["ops"]:
        if kind == S.BWD:
            assert sv == b - 1 and nv == b - 1


def test_stage_version_is_count_of_earlier_backwards_on_that_worker():
    sim = S.simulate(5, 2, 9)
    seen = [0] * 5
    for (t, s, kind, b, j, sv, nv) in sim["ops"]:
        assert sv == seen[s]
        if kind == S.BWD:
            seen[s] += 1


def test_single_worker_is_sequential():
    sim = S.simulate(1, 4, 3)
    kinds = [(op[2], op[3], op[4]) for op in sim["ops"]]
    want = []
    for b in (1, 2, 3):
        want += [(S.FWD, b, j) for j in range(4)] + [(S.BWD, b, -1)]
    assert kinds == want


def test_domain_errors():
    with pytest.raises(ValueError):
        S.version_difference_formula(1, 4)
    with pytest.raises(ValueError):
        S.simulate(0, 2, 1)


def test_stash_depth():
    # mini-batches alive at once on worker s (1-based): ceil((2(W-s)+N)/N) micro-batch groups
    for W, N in PAIRS:
        need = S.stash_groups_needed(W, N, 3 * W + 4)
        for s in range(W):
            assert need[s] == -(-(2 * (W - 1 - s) + N) // N), (W, N, s, need)
