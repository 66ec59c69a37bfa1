"""nF1B schedule by time-point simulation, with version bookkeeping.

Test infrastructure (CPU oracle); integers only.

Rules, each taken from the paper's description of its figures:
  * time is discrete and a worker performs one task per time-point (the grid
    of the workflow figures, section "Model Architecture");
  * a micro-batch forwarded by worker s at time t can be processed by worker
    s+1 from t+1 on, and a backward pass done by worker s at t reaches s-1 at
    t+1 (f_1 = W+N-1 and b = W, section "Mathematical Relationship between W
    and N");
  * worker 1 injects the next micro-batch whenever it has no backward pass to
    do; the others process forwarded micro-batches in arrival order
    (f_2 = f_1 + 1);
  * the backward pass of a mini-batch starts on the last worker right after
    the forward pass of its last micro-batch ends (section "Mathematical
    Expression for Version Difference");
  * a backward pass that has arrived is done before any waiting forward
    (section "Work Scheduling": priority on arrival);
  * the weight update of a stage follows its backward pass in the same
    time-point and is visible from the next time-point on.

Workers are numbered 0..W-1 here (worker 1 of the paper is index 0);
mini-batches are numbered from 1 as in the paper, micro-batches from 0 (A=0).
"""
from collections import deque

FWD = 0
BWD = 1


def simulate(W, N, n_minibatches):
    """Run the schedule until every mini-batch has finished its backward pass on worker 1.

    Returns a dict with
      ops: list of (t, stage, kind, b, j, stage_version, network_version) in
           (t, stage) order.  j is -1 for a backward pass.  stage_version is the
           number of updates the worker had applied before the task.
           network_version is the whole-network version of the pass the task
           belongs to: the number of mini-batches whose backward pass had left
           worker 1 strictly before the time-point at which the pass started
           (injection of the micro-batch for a forward, start on the last
           worker for a backward).
      fwd_start, fwd_end, bwd_start, bwd_end: per mini-batch time-points.
    """
    if W < 1 or N < 1 or n_minibatches < 1:
        raise ValueError("W, N and n_minibatches must be positive")
    fq = [deque() for _ in range(W)]      # (arrival, b, j)
    bq = [deque() for _ in range(W)]      # (arrival, b)
    total_micro = n_minibatches * N
    injected = 0
    stage_version = [0] * W
    net_done_times = []                   # time-points at which a backward left worker 1
    inj_version = {}
    bwd_version = {}
    fwd_start, fwd_end, bwd_start, bwd_end = {}, {}, {}, {}
    ops = []
    finished = 0
    t = 0
    while finished < n_minibatches:
        t += 1
        nv = sum(1 for tt in net_done_times if tt < t)
        for s in range(W):
            if bq[s] and bq[s][0][0] <= t:
                _, b = bq[s].popleft()
                if s == W - 1:
                    bwd_version[b] = nv
                    bwd_start[b] = t
                ops.append((t, s, BWD, b, -1, stage_version[s], bwd_version[b]))
                stage_version[s] += 1
                if s > 0:
                    bq[s - 1].append((t + 1, b))
                else:
                    net_done_times.append(t)
                    bwd_end[b] = t
                    finished += 1
                continue
            if s == 0:
                if injected >= total_micro:
                    continue
                b, j = injected // N + 1, injected % N
                injected += 1
                inj_version[(b, j)] = nv
                if j == 0:
                    fwd_start[b] = t
            else:
                if not (fq[s] and fq[s][0][0] <= t):
                    continue
                _, b, j = fq[s].popleft()
            ops.append((t, s, FWD, b, j, stage_version[s], inj_version[(b, j)]))
            if s < W - 1:
                fq[s + 1].append((t + 1, b, j))
            else:
                if j == N - 1:
                    fwd_end[b] = t
                    bq[s].append((t + 1, b))
    return {"ops": ops, "fwd_start": fwd_start, "fwd_end": fwd_end,
            "bwd_start": bwd_start, "bwd_end": bwd_end, "W": W, "N": N,
            "n_minibatches": n_minibatches}


def version_difference_simulated(W, N):
    """Steady-state version difference: index of a mini-batch minus the whole-network
    version its backward pass sees (section "Multiple Sequence Problem", Solution)."""
    n = 4 * W + 4 * N + 8
    sim = simulate(W, N, n)
    last = n
    for op in sim["ops"]:
        if op[2] == BWD and op[3] == last and op[1] == W - 1:
            return last - op[6]
    raise AssertionError("backward of the last mini-batch not found")


def version_difference_formula(W, N):
    """Final closed form of the paper for v: floor((W + N - 2) / N), domain W, N >= 2."""
    if W < 2 or N < 2:
        raise ValueError("the paper defines v for W >= 2 and N >= 2")
    return (W + N - 2) // N


def minibatches_entered_during_first_forward(W, N):
    """floor((W + N - 1) / N): mini-batches wholly injected while mini-batch 1 is in its forward pass."""
    return (W + N - 1) // N


def update_chains(W, N, n_minibatches):
    """Group mini-batches into the sequences through which an update propagates: b is
    linked to the mini-batch whose update its backward pass sees as the newest."""
    sim = simulate(W, N, n_minibatches)
    parent = {}
    for op in sim["ops"]:
        if op[2] == BWD and op[1] == W - 1:
            parent[op[3]] = op[6]          # newest whole-network version seen (0 = initial weights)
    chains = {}
    for b in sorted(parent):
        root = b
        while parent[root] != 0:
            root = parent[root]
        chains.setdefault(root, []).append(b)
    return list(chains.values())


def stash_groups_needed(W, N, n_minibatches):
    """Per worker: the largest number of mini-batches that have started their forward pass on
    that worker and not yet finished their backward pass there (activation stash depth)."""
    sim = simulate(W, N, n_minibatches)
    live = [set() for _ in range(W)]
    need = [0] * W
    for (t, s, kind, b, j, _, _) in sim["ops"]:
        if kind == FWD:
            live[s].add(b)
            need[s] = max(need[s], len(live[s]))
        else:
            live[s].discard(b)
    return need


def grid(W, N, n_minibatches, t_max=None):
    """Text rendering of the workflow figure: one row per worker, one column per time-point."""
    sim = simulate(W, N, n_minibatches)
    T = max(op[0] for op in sim["ops"])
    if t_max is not None:
        T = min(T, t_max)
    rows = [["--"] * T for _ in range(W)]
    for (t, s, kind, b, j, _, _) in sim["ops"]:
        if t <= T:
            rows[s][t - 1] = ("%d%s" % (b, chr(ord("A") + j))) if kind == FWD else ("B%d" % b)
    return rows
