"""The comparison system of the paper, PipeDream-style training, in the oracle's terms.

Test infrastructure (CPU oracle).  From the paper's account of PipeDream (related work): every batch makes its own
forward pass and its own backward pass through the W workers, a backward pass starts right after the forward pass
ends on the last worker, and workers follow 1F1B (one forward, one backward in turn once the pipeline is full) so that
forward and backward passes never wait for each other in a circle.  Horizontal weight stashing: on every worker the
backward pass of a batch reads the weights its forward pass read there, kept aside meanwhile; the gradient computed
on those stale weights is applied to the worker's current weights (the update rule of PipeDream: the gradient is taken
at weights that are W - 1 updates old on the first worker).  TiMePReSt differs in exactly two points: N forward passes
share one backward pass, and that backward pass reads the current weights, so no version is kept.

Schedule by time-point simulation, with the rules of oracle/schedule.py where they apply: one task per worker and
time-point; what a worker finishes at t reaches its neighbour at t+1; a backward pass that has arrived is done before
a waiting forward pass; worker s (from 0) makes a forward pass only while fewer than W - s batches are in flight on it
(forwarded there, backward pass still to come): the depth PipeDream fills at start-up, after which a worker takes
forward and backward passes in turn.

Workers 0..W-1, batches from 1.  The vertical weight stashing PipeDream can add (one version across workers) is not
modelled: every forward pass reads the live weights of its worker.
"""
from collections import deque

import numpy as np

from .schedule import BWD, FWD
from .stage import Stage


def simulate_1f1b(W, n_batches):
    """ops: list of (t, worker, kind, batch, -1, version_read, live_version) in (t, worker) order.  version_read:
    the number of updates in the weights the task reads (a backward pass: those of its forward pass); live_version:
    the number of updates the worker had applied before the task."""
    if W < 1 or n_batches < 1:
        raise ValueError("W and n_batches must be positive")
    fq = [deque() for _ in range(W)]
    bq = [deque() for _ in range(W)]
    live = [0] * W
    in_flight = [0] * W
    read_by_forward = {}
    admitted = done = 0
    ops = []
    t = 0
    while done < n_batches:
        t += 1
        for s in range(W):
            if bq[s] and bq[s][0][0] <= t:
                _, b = bq[s].popleft()
                ops.append((t, s, BWD, b, -1, read_by_forward[(s, b)], live[s]))
                live[s] += 1
                in_flight[s] -= 1
                if s > 0:
                    bq[s - 1].append((t + 1, b))
                else:
                    done += 1
                continue
            if in_flight[s] >= W - s:
                continue
            if s == 0:
                if admitted >= n_batches:
                    continue
                admitted += 1
                b = admitted
            else:
                if not (fq[s] and fq[s][0][0] <= t):
                    continue
                _, b = fq[s].popleft()
            in_flight[s] += 1
            read_by_forward[(s, b)] = live[s]
            ops.append((t, s, FWD, b, -1, live[s], live[s]))
            if s < W - 1:
                fq[s + 1].append((t + 1, b))
            else:
                bq[s].append((t + 1, b))
    return ops


def versions_kept(W, n_batches):
    """Per worker: the largest number of OLDER weight versions a backward pass reaches back (live - read)."""
    need = [0] * W
    for (t, s, kind, b, _, read, live) in simulate_1f1b(W, n_batches):
        if kind == BWD:
            need[s] = max(need[s], live - read)
    return need


def batches_in_flight(W, n_batches):
    """Per worker: the largest number of batches forwarded there whose backward pass is still to come (activation
    stash depth, and with the live weights the number of weight versions in use)."""
    cur, need = [0] * W, [0] * W
    for (t, s, kind, b, _, read, live) in simulate_1f1b(W, n_batches):
        cur[s] += 1 if kind == FWD else -1
        need[s] = max(need[s], cur[s])
    return need


def run_1f1b(stage_specs, params, batches, lr, momentum, precision="f64", trace=None):
    """Train len(batches) batches (x [B, ...], labels [B]) through the workers given by stage_specs / params.
    Returns dict(losses=[per batch], ops=the schedule with versions, stages=[Stage])."""
    K = len(stage_specs)
    B = len(batches[0][0])
    stages = [Stage(stage_specs[s], params[s], lr, momentum, B, 1, precision) for s in range(K)]
    ops = simulate_1f1b(K, len(batches))
    for s, st in enumerate(stages):
        st.keep_versions = max([live - read for (t, w, kind, b, _, read, live) in ops if w == s and kind == BWD] + [0])
    fwd_out, bwd_out, losses = {}, {}, {}
    for (t, s, kind, b, _, read, live) in ops:
        st = stages[s]
        assert st.version == live, "worker version differs from the simulated log"
        x_all, y_all = batches[b - 1]
        if kind == FWD:
            x = x_all if s == 0 else fwd_out.pop((b, s - 1))
            if s == K - 1:
                out, losses[b] = st.forward_micro(b, x, y_all)
            else:
                out = fwd_out[(b, s)] = st.forward_micro(b, x)
            if trace is not None:
                trace[("F", b, s)] = np.array(out)
        else:
            dy = None if s == K - 1 else bwd_out.pop((b, s + 1))
            dx = st.backward([b], dy, version=read)
            if s > 0:
                bwd_out[(b, s)] = dx
            if trace is not None:
                trace[("G", b, s)] = [None if g is None else {k: np.array(v) for k, v in g.items()} for g in st.grads]
            st.update()
    return {"losses": [float(losses[b]) for b in range(1, len(batches) + 1)], "ops": ops, "stages": stages}
