#!/usr/bin/env python3
"""Benchmark of the TiMePReSt stage-training hot path on one MI355X.

A step is one mini-batch through the whole path: on each of the K stages the N micro-batch forward
passes, the single backward pass with the latest weights and the in-place momentum update, issued
in nF1B order on K HIP streams by tmps_schedule_run.  Inputs are synthetic (seeded Gaussian inputs,
uniform labels, He-normal weights) and resident in HBM before the timed region.

Prints ONE JSON line: whole-job samples/s, the roofline of the dominant kernel class (measured
with HIP events on the kernels' own streams in a second pass of the same workload), samples/s of
every stage's own step with the device to itself (stage_steps), and the CPU oracle timed on a
bounded sample of the same workload as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def algorithmic_work(cfg, only_stage=None):
    """Per kernel class and per mini-batch: (launches, FLOPs, algorithmic bytes) from the shapes alone
    (of every stage, or of stage `only_stage` alone).

    Dense GEMMs count 2*rows*Din*Dout FLOPs and their operand/result bytes once; the update counts
    22 bytes per parameter in bf16 stages (read w, buf, g fp32; write w, buf fp32 and the bf16 copy)
    or 20 in fp32 stages."""
    asz = 2 if cfg.dtype == "bf16" else 4
    M, N, mb = cfg.M, cfg.N, cfg.micro
    work = {}

    def add(k, launches, flops, nbytes):
        a = work.setdefault(k, [0, 0.0, 0.0])
        a[0] += launches
        a[1] += flops
        a[2] += nbytes

    for si, st in enumerate(cfg.stages):
        if only_stage is not None and si != only_stage:
            continue
        P = 0
        for li, sp in enumerate(st):
            if sp["kind"] == "linear":
                din, dout, rows = sp["din"], sp["dout"], sp.get("rows", 1)
                P += din * dout + dout
                rf, rb = mb * rows, M * rows        # GEMM rows of a forward pass and of the backward pass
                osz = 4 if (li + 1 < len(st) and st[li + 1]["kind"] == "softmax_ce") else asz
                extra = (1 if sp.get("skip") else 0) + (1 if sp.get("act") == "gelu" else 0)   # residual read, z write
                add("dense_fwd", N, N * 2.0 * rf * din * dout,
                    N * (rf * din * asz + din * dout * asz + rf * dout * (osz + extra * asz)))
                add("dense_wgrad", 1, 2.0 * rb * din * dout, rb * (din + dout) * asz + (din * dout + dout) * 4)
                if not (si == 0 and li == 0):
                    add("dense_dgrad", 1, 2.0 * rb * din * dout, rb * (din + dout) * asz + din * dout * asz)
            elif sp["kind"] == "layernorm":
                d, rows = sp["d"], sp["rows"]
                P += 2 * d
                # forward: read x, write y (+ statistics); backward: read dy, x (+ joined residual gradient), write dx
                add("layernorm", N + 3, 0.0, N * mb * rows * (2 * d * asz + 8) + M * rows * (4 * d * asz + 8) + M * rows * 2 * d * asz)
            elif sp["kind"] == "attention":
                s_, d, h = sp["s"], sp["d"], sp["heads"]
                dh = d // h
                pairs = s_ * (s_ + 1) // 2          # causal: query i sees keys 0..i
                # forward: QK^T and PV; backward: QK^T, dO V^T, dV, dQ, dK: 2 and 5 products of 2*dh FLOPs per (query, key)
                add("attn_fwd", N, N * mb * h * pairs * 2.0 * dh * 2, N * mb * s_ * (4 * d * asz + h * 4))
                add("attn_bwd", 3, M * h * pairs * 2.0 * dh * 5, M * s_ * (8 * d * asz + 3 * h * 4))
            elif sp["kind"] == "embedding":
                v, s_, d = sp["vocab"], sp["s"], sp["d"]
                P += v * d + s_ * d
                add("embedding", N + 3, 0.0, N * mb * s_ * (4 + 2 * d * asz) + v * d * 4 + M * s_ * (d * asz + 4 + 8 * d) + s_ * d * 4)
            elif sp["kind"] == "conv":
                ho = (sp["h"] + 2 * sp["pad"] - sp["r"]) // sp["stride"] + 1
                wo = (sp["w"] + 2 * sp["pad"] - sp["s"]) // sp["stride"] + 1
                kk = sp["r"] * sp["s"] * sp["cin"]
                P += kk * sp["cout"] + sp["cout"]
                x_e, y_e = sp["h"] * sp["w"] * sp["cin"], ho * wo * sp["cout"]
                add("conv_fwd", N, N * 2.0 * mb * ho * wo * kk * sp["cout"], N * (mb * (x_e + y_e) * asz + kk * sp["cout"] * asz))
                add("conv_wgrad", 1, 2.0 * M * ho * wo * kk * sp["cout"], M * (x_e + y_e) * asz + kk * sp["cout"] * 4)
                if not (si == 0 and li == 0):
                    add("conv_dgrad", 1, 2.0 * M * ho * wo * kk * sp["cout"], M * (x_e + y_e) * asz + kk * sp["cout"] * asz)
            elif sp["kind"] == "affine":
                e = sp["h"] * sp["w"] * sp["c"]
                P += 2 * sp["c"]
                # the forward pass runs inside the convolution's epilogue; what is launched is the backward pass
                # (read dy and x, write dx) and the reduction of its per-slab partial sums
                add("affine", 2, 0.0, M * 3 * e * asz)
            elif sp["kind"] == "resadd":
                e = sp["h"] * sp["w"] * sp["c"]
                add("resadd", N, 0.0, N * mb * 3 * e * asz)
            elif sp["kind"] == "avgpool":
                e = sp["h"] * sp["w"] * sp["c"]
                add("pool_fwd", N, 0.0, N * mb * (e + sp["c"]) * asz)
                add("pool_bwd", 1, 0.0, M * (2 * e + sp["c"]) * asz)
            elif sp["kind"] == "maxpool":
                pad = sp.get("pad", 0)
                ho, wo = (sp["h"] + 2 * pad - sp["k"]) // sp["stride"] + 1, (sp["w"] + 2 * pad - sp["k"]) // sp["stride"] + 1
                x_e, y_e = sp["h"] * sp["w"] * sp["c"], ho * wo * sp["c"]
                add("pool_fwd", N, 0.0, N * mb * (x_e + y_e) * asz)
                add("pool_bwd", 1, 0.0, M * (2 * x_e + y_e) * asz)
            elif sp["kind"] == "softmax_ce":
                c, rows = sp["classes"], sp.get("rows", 1)
                add("softmax_ce", N, 0.0, N * mb * rows * (c * 4 + c * asz + 8))
        add("update", 1, 0.0, P * (22 if cfg.dtype == "bf16" else 20))
    return work


# classes whose kernels carry their own start/stop timestamps (no bracket overhead)
KERNEL_STAMPED = ("dense_fwd", "dense_dgrad", "dense_wgrad", "conv_fwd", "conv_dgrad", "conv_wgrad", "splitk_finish",
                  "slice_sum", "layernorm", "attn_fwd", "attn_bwd", "embedding", "affine", "resadd")


def measured_traffic(workload, kernel_class):
    """HBM bytes per launch of a kernel class from the committed counter summary
    profiles/hbm_traffic_<workload>.txt (lines `<class> <fetch bytes/launch> <write bytes/launch>`,
    already scaled by the copy-kernel factor), or None when no summary covers it."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == kernel_class:
            return float(f[1]) + float(f[2])
    return None


def stage_step_rates(T, cfg, params, steps, warmup=3):
    """Each stage of `cfg` ALONE on the device: its training step (N micro-batch forward passes, the backward pass over
    the mini-batch, the update) repeated on one stream, stash warm, fed resident synthetic boundary tensors of the
    stage's own shapes (the workload's inputs and labels on the first and last stage, Gaussian activations and
    gradients of magnitude 1/M elsewhere).  samples/s = M / time per step."""
    import numpy as np
    import torch
    from workloads import make_batch
    from workloads.configs import stage_shapes
    dev = torch.device("cuda:0")
    M, N, mb = cfg.M, cfg.N, cfg.micro
    x0, labels0 = make_batch(cfg, 0)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(cfg.seed)
    out = []
    for si in range(cfg.K):
        st = T.Stage(cfg.stages[si], cfg.dtype, mb, N, N, cfg.lr, cfg.momentum, borrow_input=True, device=dev)
        st.set_params(params[si])
        adt = st.act_dtype
        if si == 0:
            xd = st.prepare_input(x0)
        else:
            xd = torch.randn(M, st.in_elems, generator=gen).to(adt).to(dev)
        xd = xd.reshape(M, -1).contiguous()
        ld = torch.from_numpy(np.ascontiguousarray(labels0.astype(np.int32))).to(dev) if st.is_last else None
        dy = None if st.is_last else (torch.randn(M, st.out_elems, generator=gen) / M).to(adt).to(dev)
        y = None if st.is_last else torch.empty(mb * st.out_elems, dtype=adt, device=dev)
        loss = torch.zeros(1, dtype=torch.float32, device=dev) if st.is_last else None
        dx = None if si == 0 else torch.empty(M * st.in_elems, dtype=adt, device=dev)
        slots = list(range(N))

        def step():
            for j in range(N):
                st.forward_micro(j, xd[j * mb:(j + 1) * mb], y=y, labels=ld[j * mb:(j + 1) * mb] if st.is_last else None,
                                 loss_out=loss)
            st.backward(slots, dy=dy, dx=dx)
            st.update()

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        assert loss is None or bool(torch.isfinite(loss).all()), "non-finite loss on stage %d" % si
        flops = sum(v[1] for v in algorithmic_work(cfg, only_stage=si).values())
        out.append({"stage": si, "samples_per_s": M / dt, "ms_per_step": 1e3 * dt, "gflop_per_step": flops / 1e9,
                    "mfma_frac_of_bf16_peak": flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else None})
        del st, xd, dy, y, dx
    return out


def baseline_report(T, cfg, params, steps, warmup):
    """The comparison system of the paper beside the method, same workload, same number of samples: PipeDream-style
    1F1B with horizontal weight stashing in batches of the configuration's micro-batch size (one backward pass and one
    update per batch), against TiMePReSt (N forward passes, one backward pass on the live weights and one update per
    mini-batch).  Time per mini-batch's worth of samples, and the bytes every stage holds on the device."""
    import numpy as np
    import torch
    from workloads import make_batch

    def timed(pipe, batches, n):
        x, y = pipe.upload([batches[i % len(batches)] for i in range(n)])
        l = torch.zeros(n, dtype=torch.float32, device=pipe.device)
        torch.cuda.synchronize()
        pipe.run_device(x, y, max(1, min(n, warmup * (n // max(steps, 1)))), l, want_log=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipe.run_device(x, y, n, l, want_log=False)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt, bool(np.all(np.isfinite(l.cpu().numpy())))

    out = {}
    for mode in ("timeprest", "pipedream_style_1f1b"):
        base = mode != "timeprest"
        pipe = T.Pipeline(cfg, params, baseline_1f1b=base)
        per = cfg.micro if base else cfg.M
        n = steps * (cfg.N if base else 1)
        batches = [make_batch(cfg, i, M=per) for i in range(min(n, 16))]
        dt, finite = timed(pipe, batches, n)
        mem = [st.device_bytes() for st in pipe.stages]
        out[mode] = {"samples_per_s": per * n / dt, "ms_per_mini_batch_of_samples": 1e3 * dt / steps, "finite_losses": finite,
                     "backward_passes_and_updates_per_mini_batch_of_samples": cfg.N if base else 1,
                     "stage_bytes": mem, "stage_total_bytes": [sum(m.values()) for m in mem]}
        del pipe
        torch.cuda.empty_cache()
    a, b = out["timeprest"], out["pipedream_style_1f1b"]
    out["timeprest_over_baseline"] = {
        "speed": a["samples_per_s"] / b["samples_per_s"],
        "stage_memory": [x / y for x, y in zip(a["stage_total_bytes"], b["stage_total_bytes"])],
        "stage_parameter_memory": [(m["params"] + m["kept_versions"]) / (n_["params"] + n_["kept_versions"])
                                   for m, n_ in zip(a["stage_bytes"], b["stage_bytes"])],
        "paper_context": "the paper reports nearly 50 % / 40 % less GPU memory than PipeDream on stage 0 / 1 of a 2-stage "
                         "VGG-16 (its hardware, its framework, real datasets): context, not a target"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="gpt2_small_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--one-stream", action="store_true",
                    help="issue all K workers on one stream (no overlap between kernels): a diagnostic, not the metric")
    ap.add_argument("--cpu-steps", type=int, default=0, help="mini-batches the oracle is timed on (0: about 15 s worth)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy kernel (reference for scaling HBM byte counters)")
    ap.add_argument("--vertical-sync", action="store_true",
                    help="forward passes read the weight version they are tagged with (the paper's vertical weight stashing: "
                         "every stage keeps older copies of its parameters) instead of the live weights: measures what the "
                         "in-place policy of the default run saves")
    ap.add_argument("--baseline-1f1b", action="store_true",
                    help="instead of the benchmark proper: the paper's comparison system (PipeDream-style 1F1B, a backward pass "
                         "and an update per micro-batch-sized batch, backward passes on the stashed weights of their forward "
                         "passes) beside TiMePReSt on the same workload: time per mini-batch's worth of samples and per-stage bytes")
    ap.add_argument("--graphs", action="store_true",
                    help="every stage replays captured HIP graphs of its forward and backward passes (tmps_stage_use_graphs)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short throughput runs of the other benchmark configurations (reported under other_workloads)")
    ap.add_argument("--one-stream-passes", type=int, default=3,
                    help="per-kernel timing passes with all workers on one stream (the roofline figures take the lowest class "
                         "averages among them); 0: none, the roofline then shows the K-stream durations")
    ap.add_argument("--hw-queues", type=int, default=8,
                    help="hardware queues HIP may use (GPU_MAX_HW_QUEUES, read when HIP starts): the K stage streams and "
                         "the default stream share the runtime's default of 4, so two stages would take turns on one queue")
    args = ap.parse_args()
    if args.hw_queues > 0:   # before anything initialises HIP
        os.environ["GPU_MAX_HW_QUEUES"] = str(min(args.hw_queues, 32))
    if args.gpus != 1:
        print("bench.py: this build runs the stage-training path on ONE GPU (K stages on K streams of the same "
              "device); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2410_14312_amd as T
    from workloads import get_config, init_params, make_batch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)          # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    cfg = get_config(args.workload)
    params = init_params(cfg)
    if args.baseline_1f1b:
        rep = baseline_report(T, cfg, params, args.steps, args.warmup)
        print(json.dumps({"metric": "training samples/sec per stage on 1 MI355X: TiMePReSt beside the PipeDream-style baseline",
                          "unit": "samples/s", "value": rep["timeprest"]["samples_per_s"], "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
                          "config": {"workload": cfg.name, "mini_batch": cfg.M, "micro_batches": cfg.N, "stages": cfg.K},
                          "comparison": rep}))
        return
    pipe = T.Pipeline(cfg, params, one_stream=args.one_stream, vertical_sync=args.vertical_sync, graphs=args.graphs)
    shadow_bytes = sum(int(st.shadow.numel()) for st in pipe.stages if getattr(st, "shadow", None) is not None)
    n_distinct = min(32, max(args.steps, args.warmup, 1))
    distinct = [make_batch(cfg, i) for i in range(n_distinct)]

    def resident(n):
        x, y = pipe.upload([distinct[i % n_distinct] for i in range(n)])
        return x, y, torch.zeros(n, dtype=torch.float32, device=pipe.device)

    xw, yw, lw = resident(max(args.warmup, 1))
    xs, ys, ls = resident(args.steps)
    torch.cuda.synchronize()
    if args.warmup > 0:
        pipe.run_device(xw, yw, args.warmup, lw, want_log=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.run_device(xs, ys, args.steps, ls, want_log=False)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    losses = ls.cpu().numpy()
    # (under vertical weight stashing the convolutional configurations diverge at their configured learning rate, in
    # the oracle as on the GPU: the throughput of that mode is reported all the same, with the fact)
    diverged = not bool(np.all(np.isfinite(losses)))
    assert args.vertical_sync or not diverged, "non-finite loss in the timed run"
    value = cfg.M * args.steps / dt

    work = algorithmic_work(cfg)

    def timed_pass(one_stream):
        """The same workload once more with per-kernel timing on the kernels' streams; per-class summary."""
        T.profile_enable(True)
        pipe.run_device(xs, ys, args.steps, ls, want_log=False, one_stream=one_stream)
        torch.cuda.synchronize()
        prof = T.profile_read()
        T.profile_enable(False)
        out = []
        # what an empty pair of timing events measures on these streams; subtracted from every bracket
        pair_ms, pair_cnt = prof.pop("event_pair", (0.0, 0))
        pair_us = 1e3 * pair_ms / pair_cnt if pair_cnt else 0.0
        for k, (ms, cnt) in prof.items():
            if cnt == 0:
                continue
            per = work.get(k)
            if k not in KERNEL_STAMPED:      # bracketed classes also contain the cost of the event pair
                ms = max(ms - cnt * pair_us / 1e3, 0.05 * ms)
            ent = {"class": k, "launches_per_step": cnt / args.steps, "avg_us": 1e3 * ms / cnt, "ms_per_step": ms / args.steps}
            if per and per[0]:
                ent["gflop_per_launch"] = per[1] / per[0] / 1e9
                ent["mbytes_per_launch"] = per[2] / per[0] / 1e6
                sec = ms / cnt / 1e3
                ent["tflops"] = per[1] / per[0] / sec / 1e12
                ent["gbs"] = per[2] / per[0] / sec / 1e9
            out.append(ent)
        out.sort(key=lambda e: -e["ms_per_step"])
        return out, pair_us

    # Pass 2: the benchmark's own configuration (K streams): while kernels of several stages share the device, each
    # takes longer than it would alone, so these durations describe the mix, not the kernels.
    kernels, pair_us = timed_pass(args.one_stream)
    # Pass 3: every worker on one stream, so each kernel has the device to itself: the per-kernel rates that the
    # roofline is about.
    # (three such passes, per class the one with the lowest average: a pass during which the host stalls or the clocks
    # still ramp reads several microseconds high on every launch)
    if args.one_stream or args.one_stream_passes <= 0:
        kernels_alone, pair_us_alone = kernels, pair_us
    else:
        passes = [timed_pass(True) for _ in range(args.one_stream_passes)]
        pair_us_alone = min(p[1] for p in passes)
        best = {}
        for plist, _ in passes:
            for e in plist:
                if e["class"] not in best or e["avg_us"] < best[e["class"]]["avg_us"]:
                    best[e["class"]] = e
        kernels_alone = sorted(best.values(), key=lambda e: -e["ms_per_step"])
    dom = kernels_alone[0]
    hbm_bound = dom["class"] in ("update", "softmax_ce", "pool_fwd", "pool_bwd", "relu_mask", "copy", "reduce", "layernorm",
                                 "embedding", "affine", "resadd")
    peak = HBM_PEAK_GBS if hbm_bound else (MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else 157.3)
    rate = "gbs" if hbm_bound else "tflops"
    roof = {"kernel": dom["class"], "bound": "hbm" if hbm_bound else "mfma", "achieved": dom.get(rate, 0.0), "peak": peak,
            "unit": "GB/s" if hbm_bound else "TFLOP/s", "frac": dom.get(rate, 0.0) / peak,
            "traffic": measured_traffic(cfg.name, dom["class"]), "avg_launch_us": dom["avg_us"],
            "launches_per_step": dom["launches_per_step"],
            "timing": "per-launch durations of a pass of the same mini-batches with all workers on one stream (no other "
                      "kernel on the device; per class the lowest average of such passes); rocprofv3 summary of "
                      "that command: profiles/%s_one_stream_kernel_trace.txt" % cfg.name,
            "event_pair_us_subtracted": pair_us_alone}
    shared = next((e for e in kernels if e["class"] == dom["class"]), None)
    if shared is not None and not args.one_stream:
        roof["with_%d_streams" % cfg.K] = {"avg_launch_us": shared["avg_us"], "achieved": shared.get(rate, 0.0),
                                          "frac": shared.get(rate, 0.0) / peak}

    flops_step = sum(v[1] for v in work.values())
    cpu = None
    if not args.no_cpu_baseline:
        cores = len(os.sched_getaffinity(0))
        if flops_step > 1e12 and args.cpu_steps <= 0:
            # A whole mini-batch through the fp64 oracle would take minutes: time ONE stage's step instead
            # (N micro-batch forward passes, the backward pass, the update) on an inner stage of the same
            # workload, fed Gaussian activations of that stage's input shape.
            from oracle.stage import Stage as OStage
            from workloads.configs import stage_shapes
            from workloads import to_bf16_grid
            si = 1 if cfg.K > 2 else 0
            in_shape, out_shape = stage_shapes(cfg)[si]
            rng = np.random.default_rng(cfg.seed)
            if si == 0 and cfg.vocab:
                xin = distinct[0][0]
            else:
                xin = to_bf16_grid(rng.standard_normal((cfg.M, int(np.prod(in_shape)))).astype(np.float32))
            dy = to_bf16_grid((rng.standard_normal((cfg.M, int(np.prod(out_shape)))) / cfg.M).astype(np.float32))
            ost = OStage(cfg.stages[si], params[si], cfg.lr, cfg.momentum, cfg.M, cfg.N,
                         precision="bf16" if cfg.dtype == "bf16" else "f64")
            t1 = time.perf_counter()
            for j in range(cfg.N):
                ost.forward_micro(j, xin[j * cfg.micro:(j + 1) * cfg.micro])
            ost.backward(list(range(cfg.N)), dy)
            ost.update()
            dc = time.perf_counter() - t1
            cpu = {"value": cfg.M / dc, "unit": "samples/s", "cores": cores, "kind": "oracle", "stage": si,
                   "sample": "one training step (N forward passes, backward pass, update) of stage %d of %d alone (its "
                             "layers only: samples/s of that stage, not of the whole pipeline) through the numpy fp64 "
                             "oracle (%.1f s)" % (si, cfg.K, dc)}
        else:
            from oracle import pipeline as opipe
            n_cpu = args.cpu_steps
            if n_cpu <= 0:
                t1 = time.perf_counter()
                opipe.run(cfg, params, distinct[:2])
                per = (time.perf_counter() - t1) / 2
                n_cpu = int(max(2, min(n_distinct, 15.0 / max(per, 1e-3))))
            t1 = time.perf_counter()
            opipe.run(cfg, params, distinct[:n_cpu])
            dc = time.perf_counter() - t1
            cpu = {"value": cfg.M * n_cpu / dc, "unit": "samples/s", "cores": cores, "kind": "oracle", "stage": None,
                   "sample": "%d mini-batches of the same workload through the numpy fp64 oracle pipeline (%.1f s)" % (n_cpu, dc)}

    # Every stage's own training step with the device to itself (one stream, no other stage's kernels).
    del pipe, xw, yw, lw, xs, ys, ls
    torch.cuda.empty_cache()
    stage_steps = None
    if not args.one_stream and not args.calibrate_copy and not args.vertical_sync:
        stage_steps = stage_step_rates(T, cfg, params, max(5, min(args.steps, 20)))
    # The other benchmark configurations, for context: the same measurement (resident inputs, K streams, wall time
    # between device synchronisations) on a short run each, without per-kernel timing, and their stages' own steps.
    others = []
    if not args.no_other_workloads and not args.one_stream and not args.calibrate_copy and not args.vertical_sync:
        for name in ("tiny_mlp_f32", "mlp4x1024_bf16", "vgg16_bf16", "resnet50_bf16", "gpt2_small_bf16"):
            if name == cfg.name:
                continue
            ocfg = get_config(name)
            oparams = init_params(ocfg)
            opipe_ = T.Pipeline(ocfg, oparams, graphs=args.graphs)
            n = 20 if name in ("resnet50_bf16", "gpt2_small_bf16") else 60
            ob = [make_batch(ocfg, i) for i in range(min(n, 8))]
            ox, oy = opipe_.upload([ob[i % len(ob)] for i in range(n)])
            ol = torch.zeros(n, dtype=torch.float32, device=opipe_.device)
            torch.cuda.synchronize()
            opipe_.run_device(ox, oy, n, ol, want_log=False)   # warm-up pass
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            opipe_.run_device(ox, oy, n, ol, want_log=False)
            torch.cuda.synchronize()
            od = time.perf_counter() - t1
            assert np.all(np.isfinite(ol.cpu().numpy())), "non-finite loss in %s" % name
            ow = algorithmic_work(ocfg)
            del opipe_, ox, oy, ol
            torch.cuda.empty_cache()
            others.append({"workload": name, "value": ocfg.M * n / od, "unit": "samples/s", "ms_per_step": 1e3 * od / n,
                           "steps": n, "mini_batch": ocfg.M, "micro_batches": ocfg.N, "stages": ocfg.K,
                           "dtype": "bf16" if ocfg.dtype == "bf16" else "f32",
                           "mfma_frac_of_bf16_peak_end_to_end": (sum(v[1] for v in ow.values()) / (od / n) / 1e12 / MFMA_BF16_PEAK_TFLOPS)
                           if ocfg.dtype == "bf16" else None,
                           "stage_steps": stage_step_rates(T, ocfg, oparams, 20)})

    if cpu is not None:
        if cpu.get("stage") is not None and stage_steps:
            # like for like: the same stage's step on the GPU, the device to itself
            cpu["gpu_same_sample"] = {"value": stage_steps[cpu["stage"]]["samples_per_s"], "unit": "samples/s",
                                      "what": "training step of stage %d alone on the GPU (stage_steps[%d])" % (cpu["stage"], cpu["stage"])}
        elif cpu.get("stage") is None:
            cpu["gpu_same_sample"] = {"value": value, "unit": "samples/s", "what": "the whole pipeline (value)"}
    out = {
        # every stage of the pipeline processes every sample, so the pipeline's rate IS each stage's rate in it; the
        # rate each stage reaches with the device to itself is under stage_steps
        "metric": "training samples/sec per stage on 1 MI355X; MFMA util % of bf16 peak",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "mini_batch": cfg.M, "micro_batches": cfg.N, "stages": cfg.K,
                   "measured": "K stages in nF1B order on K streams of one GPU (every stage processes every sample)",
                   "version_difference": T.version_diff_simulated(cfg.K, cfg.N),
                   "weight_policy": "vertical weight stashing" if args.vertical_sync else "in place",
                   "shadow_weight_bytes": shadow_bytes,
                   "streams": 1 if args.one_stream else cfg.K, "hw_queues": int(os.environ.get("GPU_MAX_HW_QUEUES", "4")),
                   "graphs": bool(args.graphs)},
        "mfma_frac_of_bf16_peak_end_to_end": flops_step / (dt / args.steps) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "stage_steps": stage_steps, "roofline": roof, "cpu_baseline": cpu, "kernels": kernels, "kernels_one_stream": kernels_alone,
        "final_loss": float(losses[-1]) if np.isfinite(losses[-1]) else None, "diverged": diverged, "other_workloads": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
