"""K workers of the CPU oracle driven by the simulated nF1B schedule.

Test infrastructure (CPU oracle).  Tasks are executed in time-point order;
within a time-point the workers do not interact (what one produces reaches its
neighbour at the next time-point), so the order inside a time-point is free.
Each worker reads and updates only its own weights, in place: a forward pass
sees whatever the worker's weights are when the micro-batch gets there, and a
backward pass the weights at that moment.
"""
import numpy as np

from . import schedule as S
from .stage import Stage


def run(cfg, params, batches, trace=None, precision=None, momentum=None, versions=None, vertical_sync=False):
    """Train `len(batches)` mini-batches.

    cfg: a workloads.Config (shape tables only); params: per stage, per layer dicts of arrays;
    batches: list of (x [M, ...], labels [M]).  precision: storage policy ("f64" or "bf16", see
    oracle/precision.py); by default the one the configuration names.  trace: optional dict that receives every task's
    tensors under (kind, b, j, stage) keys.
    vertical_sync: the paper's own weight policy for forward passes (Methodology, first paragraph: vertical weight
    stashing keeps a forward pass on one weight version across all workers).  A micro-batch is tagged with the
    number of whole-network updates completed when it enters worker 1 (the log's last field), and every later worker
    runs its forward pass on ITS weights after that many updates, which it keeps until no forward pass needs them
    ("GPU Memory Overhead").  Backward passes read the live weights either way.  False: every task reads the live
    weights of its worker (no stashed versions).
    momentum, versions: state to resume from (section "Checkpointing": a run restarts from the parameters every
    stage saved at the end of an epoch; with momentum the buffers and the update counters belong to that state):
    per stage, per layer dicts like params, and per stage update counts.  The version log of a resumed run counts
    from zero again.
    Returns dict(losses=[per mini-batch mean of the micro-batch losses], ops=version log,
    stages=[Stage]).
    """
    K, N, M = cfg.K, cfg.N, cfg.M
    micro = M // N
    if precision is None:
        precision = "bf16" if cfg.dtype == "bf16" else "f64"
    stages = [Stage(cfg.stages[s], params[s], cfg.lr, cfg.momentum, M, N, precision) for s in range(K)]
    if momentum is not None:
        for st, bufs in zip(stages, momentum):
            st.bufs = [{k: np.array(v, dtype=np.float64) for k, v in b.items()} for b in bufs]
    base = [0] * K if versions is None else [int(v) for v in versions]
    for st, v in zip(stages, base):
        st.version = v
    sim = S.simulate(K, N, len(batches))
    if vertical_sync:
        for s_, st in enumerate(stages):
            st.keep_versions = max([sv - nv for (t, w, kind, b, j, sv, nv) in sim["ops"] if kind == S.FWD and w == s_] + [0])
    fwd_out = {}
    bwd_out = {}
    micro_losses = {}
    for (t, s, kind, b, j, sv, nv) in sim["ops"]:
        st = stages[s]
        assert st.version - base[s] == sv, "worker version differs from the simulated log"
        if kind == S.FWD:
            x_all, y_all = batches[b - 1]
            if s == 0:
                x = x_all[j * micro:(j + 1) * micro]
            else:
                x = fwd_out.pop((b, j, s - 1))
            ver = base[s] + nv if vertical_sync else None
            if s == K - 1:
                logits, loss = st.forward_micro((b, j), x, y_all[j * micro:(j + 1) * micro], version=ver)
                micro_losses.setdefault(b, []).append(loss)
                out = logits
            else:
                out = st.forward_micro((b, j), x, version=ver)
                fwd_out[(b, j, s)] = out
            if trace is not None:
                trace[("F", b, j, s)] = np.array(out)
        else:
            slots = [(b, jj) for jj in range(N)]
            dy = None if s == K - 1 else bwd_out.pop((b, s + 1))
            dx = st.backward(slots, dy)
            if s > 0:
                bwd_out[(b, s)] = dx
            if trace is not None:
                trace[("B", b, -1, s)] = np.array(dx)
                trace[("G", b, -1, s)] = [None if g is None else {k: np.array(v) for k, v in g.items()}
                                          for g in st.grads]
            st.update()
    losses = [float(np.mean(micro_losses[b])) for b in range(1, len(batches) + 1)]
    return {"losses": losses, "ops": sim["ops"], "stages": stages}
