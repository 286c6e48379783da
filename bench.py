#!/usr/bin/env python3
"""Benchmark of the forward + BPTT hot path on one MI355X.

A step is one pass of the whole hot path over one window of seeded synthetic input:
rnn_forward + rnn_bptt + rnn_grads (all weight gradients), with inputs / targets / weights already
resident in HBM.  Prints ONE JSON line: frames/s of the headline workload, the roofline record of
the dominant kernel (the persistent recurrent-step kernel, timed live with HIP events on the launch
stream), the float64 oracle timed on the host cores on a bounded sample of the same workload, and
under "also" short runs of the many-stream workloads (the N = 32 half of the metric and the
batched-GEMM figures against the fp32 matrix peak).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload speech_n1] [--no-cpu-baseline]
                    [--no-framewise] [--no-also] [--no-paper-schedule] [--index-input]

Workloads: speech_n1 (default: 2 x 256 peephole LSTM, T = 1024, N = 1), charlm_n1, charlm_n32,
generalized_n64, tiny; the paper's Section 4 shapes lm_elman_n1, lm_lstm_n1 (38,000-512-20,000,
T = 2048) and fig4_h{1024,2048,4096}_n{1,16,64} (all layers equally wide, mini-batch 1,024 frames).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MFMA_PEAK_TFLOPS = 157.3  # MI355X published dense fp32 matrix peak
PROF = dict(step_fwd=0, step_bwd=1, gemm_fwd=2, gemm_bwd=3, gemm_grad=4, other=5)


def recurrent_bytes_per_step(spec, sched):
    """Algorithmic bytes per time step and direction under the canonical schedule: every weight of a
    connection inside a recurrent node is touched once per step (full matrices and diagonal
    vectors), 4 bytes each."""
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
    import workloads as wl
    from oracle import graph_oracle as go
    w = wl.make_config(name, T=T_sample)
    warm = wl.make_config("tiny")
    go.forward_bptt(warm.spec.nodes, warm.spec.edges, warm.weights, warm.biases, warm.inputs, warm.targets, warm.T, warm.N)
    t0 = time.perf_counter()
    reps = 0
    while True:       # whole passes over the sample until about 10 s of CPU work have been timed
        go.forward_bptt(w.spec.nodes, w.spec.edges, w.weights, w.biases, w.inputs, w.targets, w.T, w.N)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 50:
            break
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=reps * w.T * w.N / dt, unit="frames/s", cores=int(threads), kind="oracle",
                sample=f"{name}: first {w.T} of the window's frames x {w.N} streams, {reps} forward+BPTT passes in float64 numpy, {dt:.1f} s")


def load_traffic(workload):
    """HBM bytes per step-kernel launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    try:
        with open(path) as f:
            return json.load(f)["hbm_bytes_per_launch"]
    except Exception:
        return None


def measure(name, steps, warmup, index_input=False, calibrate_copy=False):
    """Times `steps` passes of the hot path on workload `name`.  Returns the record's fields."""
    import torch
    import workloads as wl
    from paper_1503_02852_amd.runner import window_for

    w = wl.make_config(name)
    win = window_for(w, "cuda:0")
    if index_input:
        idx = {}
        for k, x in w.inputs.items():
            if not ((x == 0) | (x == 1)).all() or not (x.sum(axis=2) <= 1).all():
                print(f"bench.py: --index-input needs one-hot input frames; input node {k} of {name} is dense", file=sys.stderr)
                sys.exit(2)
            idx[k] = np.where(x.sum(axis=2) > 0, x.argmax(axis=2), -1)
        win.set_onehot_inputs(idx)
    sched = win.g.schedule()
    win.g.specialise(w.N)
    for _ in range(max(1, warmup)):
        win.step()
    win.check()          # waits; raises if a kernel flagged an error
    if calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    # timed region: K steps; HIP events only around the dominant class (the step kernels)
    win.g.profile_enable((1 << PROF["step_fwd"]) | (1 << PROF["step_bwd"]))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        win.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_f, n_f = win.g.profile_read(PROF["step_fwd"])
    ms_b, n_b = win.g.profile_read(PROF["step_bwd"])
    win.g.profile_enable(0)
    # the timed windows' results must be valid: loss read-back + error flags of the last window
    loss = win.compute_grads(want_loss=True)
    if not np.isfinite(loss):
        raise RuntimeError(f"{name}: the loss of the last timed window is not finite")

    # class breakdown in a second, separately timed pass (events around every class)
    reps = max(1, min(steps, 5))
    win.g.profile_enable(0x3F)
    for _ in range(reps):
        win.step()
    torch.cuda.synchronize()
    breakdown = {}
    for nm, cls in PROF.items():
        ms, n = win.g.profile_read(cls)
        breakdown[nm] = dict(ms_per_step=ms / reps, launches_per_step=n / reps)
    win.g.profile_enable(0)

    frames = w.T * w.N
    ms_per_step = dt * 1e3 / steps
    value = frames * steps / dt
    # what the executed plan batched and what it stepped (stacked recurrent nodes that share a step
    # launch step the connections between them: their bytes and flops belong to the step kernel)
    flops, step_bytes = win.g.plan_work(w.T, w.N)
    build_f, build_b, chained = "none", "none", False
    for k in range(len(w.spec.nodes)):           # the last recurrent node's builds (all layers of these stacks agree)
        bf, ch = win.g.step_build(k, False)
        if bf != "none":
            build_f, chained, build_b = bf, ch, win.g.step_build(k, True)[0]

    # Roofline of the dominant kernel: the persistent recurrent-step kernel.  One launch runs all T
    # steps of the recurrent nodes it covers in one direction; its algorithmic bytes are the weight
    # bytes its steps touch, once per step.
    n_launch = (n_f + n_b) / steps
    window_bytes = (step_bytes["step_fwd"] + step_bytes["step_bwd"]) * w.T
    canonical_bytes = recurrent_bytes_per_step(w.spec, sched) * w.T * 2
    loop_ms = (ms_f + ms_b) / steps
    avg_launch_ms = loop_ms / n_launch if n_launch else 0.0
    achieved = window_bytes / (loop_ms * 1e-3) / 1e9 if loop_ms > 0 else 0.0
    step_tflops = (flops["step_fwd"] + flops["step_bwd"]) / (loop_ms * 1e-3) / 1e12 if loop_ms > 0 else 0.0
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBS, unit="GB/s", frac=achieved / HBM_PEAK_GBS,
                    traffic=load_traffic(name),
                    kernel="rnng_step_jit (persistent recurrent-step kernel, forward and backward launches)",
                    algorithmic_bytes_per_launch=window_bytes / n_launch if n_launch else 0,
                    avg_launch_ms=avg_launch_ms, launches_per_window=n_launch,
                    us_per_step_of_a_launch=avg_launch_ms * 1e3 / w.T if w.T else 0.0,
                    # the same time against the bytes of the canonical schedule's recurrent nodes alone
                    # (connections between stacked layers counted as batched, whoever computes them)
                    frac_recurrent_weights_only=canonical_bytes / (loop_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if loop_ms > 0 else 0.0,
                    step_tflops=step_tflops, step_frac_of_fp32_mfma_peak=step_tflops / FP32_MFMA_PEAK_TFLOPS)

    # batched edge GEMMs against the fp32 MFMA peak: the products the executed plan batched
    gemms = {}
    for k in ("gemm_fwd", "gemm_bwd", "gemm_grad"):
        ms = breakdown[k]["ms_per_step"]
        tf = flops[k] / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        gemms[k] = dict(gflop_per_window=flops[k] / 1e9, tflops=tf, frac_of_fp32_mfma_peak=tf / FP32_MFMA_PEAK_TFLOPS)

    return dict(w=w, win=win, value=value, ms_per_step=ms_per_step, frames=frames, breakdown=breakdown, gemms=gemms,
                roofline=roofline, loss=loss, schedule="chain" if chained else "paper", step_builds=[build_f, build_b])


def short_record(m):
    """What an "also" entry keeps of a measurement."""
    w = m["w"]
    return dict(workload=w.name, T=w.T, N=w.N, value=m["value"], unit="frames/s", ms_per_step=m["ms_per_step"],
                schedule=m["schedule"], step_builds=m["step_builds"],
                paper_rule_gflops=paper_rule_flops_per_frame(w.spec) * m["frames"] / (m["ms_per_step"] * 1e-3) / 1e9,
                step_kernels=dict(ms_per_step=m["breakdown"]["step_fwd"]["ms_per_step"] + m["breakdown"]["step_bwd"]["ms_per_step"],
                                  frac_of_hbm_peak=m["roofline"]["frac"], frac_of_fp32_mfma_peak=m["roofline"]["step_frac_of_fp32_mfma_peak"],
                                  traffic=m["roofline"]["traffic"], algorithmic_bytes_per_launch=m["roofline"]["algorithmic_bytes_per_launch"]),
                batched_gemms=m["gemms"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="speech_n1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-framewise", action="store_true",
                    help="skip the frame-by-frame schedule (the paper's baseline: no batching over frames)")
    ap.add_argument("--no-also", action="store_true", help="skip the short runs of the many-stream workloads")
    ap.add_argument("--no-paper-schedule", action="store_true",
                    help="skip the extra run on Section 3.1's schedule verbatim (its step launches carry the same kernel name: profiles)")
    ap.add_argument("--index-input", action="store_true",
                    help="give one-hot input layers as class indices (column gather / scatter-add instead of GEMMs "
                         "over one-hot matrices); for the word-input workloads lm_*")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path would shard over streams with one gradient "
              "all-reduce per window, which is not built. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1503_02852_amd.runner import window_for

    m = measure(args.workload, args.steps, args.warmup, args.index_input, args.calibrate_copy)
    w, value, frames = m["w"], m["value"], m["frames"]
    out = dict(metric="forward+BPTT frames/sec (fp32)", value=value, unit="frames/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=m["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="f32", data="synthetic",
               config=dict(workload=args.workload, input="class indices" if args.index_input else "dense", T=w.T, N=w.N,
                           nodes=len(w.spec.nodes), edges=len(w.spec.edges), params=w.n_params(), frames_per_window=frames,
                           # "chain": stacked recurrent layers share one step launch and the connections between them
                           # are stepped with it; "paper": Section 3.1 verbatim, those connections batched over frames
                           schedule=m["schedule"], step_builds=m["step_builds"]),
               paper_rule_gflops=paper_rule_flops_per_frame(w.spec) * frames / (m["ms_per_step"] * 1e-3) / 1e9,
               breakdown=m["breakdown"], batched_gemms=m["gemms"], roofline=m["roofline"])
    del m
    if out["config"]["schedule"] == "chain" and not args.no_paper_schedule:
        # the same workload on the paper's schedule verbatim (one step launch per recurrent node)
        os.environ["RNNG_CHAIN"] = "0"
        try:
            p = measure(args.workload, max(3, args.steps // 4), 1, args.index_input)
        finally:
            del os.environ["RNNG_CHAIN"]
        out["paper_schedule"] = dict(value=p["value"], unit="frames/s", ms_per_step=p["ms_per_step"], schedule=p["schedule"],
                                     roofline_frac=p["roofline"]["frac"], batched_gemms=p["gemms"])
        del p
    if not args.no_framewise:
        # Section 4's baseline on the same kernels' per-frame forms: every frame on its own, no batching
        # over frames, no persistent step kernel.  Reported next to the paper's ">10x" for its own schedule.
        os.environ["RNNG_SCHEDULE"] = "framewise"
        try:
            win_fw = window_for(w, "cuda:0")
        finally:
            del os.environ["RNNG_SCHEDULE"]
        win_fw.step()
        torch.cuda.synchronize()
        reps_fw = 2
        t0 = time.perf_counter()
        for _ in range(reps_fw):
            win_fw.step()
        torch.cuda.synchronize()
        dt_fw = (time.perf_counter() - t0) / reps_fw
        out["framewise_schedule"] = dict(value=frames / dt_fw, unit="frames/s", ms_per_step=dt_fw * 1e3,
                                         speedup_of_default_schedule=value / (frames / dt_fw))
        del win_fw
    if not args.no_also and args.workload == "speech_n1":
        out["also"] = []
        for name, steps in (("charlm_n32", 10), ("generalized_n64", 5)):
            a = measure(name, steps, 2)
            out["also"].append(short_record(a))
            del a
            torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        T_sample = {"tiny": 20, "speech_n1": 1024, "charlm_n1": 512, "charlm_n32": 256, "generalized_n64": 16,
                    "lm_elman_n1": 256, "lm_lstm_n1": 256}.get(args.workload, 16)
        out["cpu_baseline"] = cpu_baseline(args.workload, T_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
