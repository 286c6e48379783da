#!/usr/bin/env python3
"""Benchmark of the forward + BPTT hot path on one MI355X.

A step is one pass of the whole hot path over one window of seeded synthetic input:
rnn_forward + rnn_bptt + rnn_grads (all weight gradients), inputs / targets / weights already
resident in HBM.  Prints ONE JSON line: frames/s, the roofline record of the dominant kernel
(recurrent-node step kernels, timed live with HIP events on the launch stream) and the float64
oracle timed on the host cores on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload speech_n1] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix peak


def recurrent_bytes_per_step(spec, sched):
    """Algorithmic bytes per time step and direction: every weight of a connection inside a
    recurrent node is touched once per step (full matrices and diagonal vectors)."""
    total = 0
    for m, e in enumerate(spec.edges):
        if sched["edge_class"][m] == 0:
            continue
        ns, nd = spec.nodes[e["src"]]["dim"], spec.nodes[e["dst"]]["dim"]
        total += 4 * (nd * ns if e["wkind"] == 0 else nd if e["wkind"] == 1 else 0)
    return total


def paper_rule_flops_per_frame(spec):
    """The paper's counting rule (Section 4): only parameter products and error-gradient
    products: 6 flops per full-edge weight per frame, 4 if the edge leaves an input node."""
    fl = 0
    for e in spec.edges:
        if e["wkind"] != 0:
            continue
        w = spec.nodes[e["src"]]["dim"] * spec.nodes[e["dst"]]["dim"]
        fl += (4 if spec.nodes[e["src"]]["kind"] == 0 else 6) * w
    return fl


def cpu_baseline(name, T_sample):
    """The oracle as it stands on a bounded sample: the same network and stream count over the
    first T_sample frames of the window."""
    import numpy as np  # noqa: F401
    import workloads as wl
    from oracle import graph_oracle as go
    w = wl.make_config(name, T=T_sample)
    warm = wl.make_config("tiny")
    go.forward_bptt(warm.spec.nodes, warm.spec.edges, warm.weights, warm.biases, warm.inputs, warm.targets, warm.T, warm.N)
    t0 = time.perf_counter()
    go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=w.T * w.N / dt, unit="frames/s", cores=int(threads), kind="oracle",
                sample=f"{name}: first {w.T} of the window's frames x {w.N} streams, one forward+BPTT in float64 numpy, {dt:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="speech_n1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path shards over streams with one gradient "
              "all-reduce per window, which is described in DESIGN.md and not built. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_1503_02852_amd.runner import window_for

    w = wl.make_config(args.workload)
    win = window_for(w, "cuda:0")
    sched = win.g.schedule()
    for _ in range(args.warmup):
        win.step()
    torch.cuda.synchronize()

    PROF_STEP_FWD, PROF_STEP_BWD, PROF_GEMM_FWD, PROF_GEMM_BWD, PROF_GEMM_GRAD, PROF_OTHER = range(6)
    win.g.profile_enable((1 << PROF_STEP_FWD) | (1 << PROF_STEP_BWD))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        win.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_f, n_f = win.g.profile_read(PROF_STEP_FWD)
    ms_b, n_b = win.g.profile_read(PROF_STEP_BWD)
    win.g.profile_enable(0)

    # class breakdown in a second, separately timed pass (events around every class)
    win.g.profile_enable(0x3F)
    for _ in range(max(1, min(args.steps, 5))):
        win.step()
    torch.cuda.synchronize()
    reps = max(1, min(args.steps, 5))
    breakdown = {}
    for cls, nm in enumerate(["step_fwd", "step_bwd", "gemm_fwd", "gemm_bwd", "gemm_grad", "other"]):
        ms, n = win.g.profile_read(cls)
        breakdown[nm] = dict(ms_per_step=ms / reps, launches_per_step=n / reps)
    win.g.profile_enable(0)

    frames = w.T * w.N
    ms_per_step = dt * 1e3 / args.steps
    value = frames * args.steps / dt

    # Roofline of the dominant kernel class: the recurrent-node step loops (both directions).
    # One "launch" here is one time step of one direction over all recurrent nodes' layers is
    # not meaningful across layers of different width, so the unit is the window: algorithmic
    # bytes = (bytes per step, all recurrent nodes) x T x 2 directions; duration = the summed
    # step-loop time per window measured by the events above.
    step_bytes = recurrent_bytes_per_step(w.spec, sched)
    window_bytes = step_bytes * w.T * 2
    loop_ms = (ms_f + ms_b) / args.steps
    achieved = window_bytes / (loop_ms * 1e-3) / 1e9 if loop_ms > 0 else 0.0
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=None, kernel="recurrent step loops (forward + backward)",
                    algorithmic_bytes_per_window=window_bytes, loop_ms_per_window=loop_ms,
                    launches_per_window=(n_f + n_b) / args.steps)

    flops = paper_rule_flops_per_frame(w.spec) * frames
    out = dict(metric="forward+BPTT frames/sec (fp32)", value=value, unit="frames/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="f32", data="synthetic",
               config=dict(workload=args.workload, T=w.T, N=w.N, nodes=len(w.spec.nodes), edges=len(w.spec.edges),
                           params=w.n_params(), frames_per_window=frames),
               paper_rule_gflops=flops / (ms_per_step * 1e-3) / 1e9,
               breakdown=breakdown, roofline=roofline)
    if not args.no_cpu_baseline:
        T_sample = {"tiny": 20, "speech_n1": 1024, "charlm_n1": 512, "charlm_n32": 128, "generalized_n64": 8}[args.workload]
        out["cpu_baseline"] = cpu_baseline(args.workload, T_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
