#!/usr/bin/env python3
"""Benchmark of the fused Signum + majority-vote step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3]

A step is one ss_signum_vote_step call over all M workers (momentum, sign,
vote, parameter update in one pass) on synthetic gradients already resident in
HBM.  The headline workload is C3: d = 25,557,032 fp32 parameters, M = 7,
beta = 0.9.  Prints ONE JSON line: params/s, the HBM roofline of the step
kernel (algorithmic bytes / measured kernel time against 8 TB/s), and the CPU
oracle timed on this machine's host cores as a baseline.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "fused_step_C3_hbm_traffic.md")


def algorithmic_bytes_per_coordinate(cfg):
    """What the method itself must move per coordinate and step: per worker read
    g and m and write m; read and write x; write one voted bit."""
    gbytes = 4 if cfg.grad_dtype == "f32" else 2
    per_worker = gbytes + (8 if cfg.beta is not None else 0)
    return cfg.M * per_worker + 8 + 0.125


def measured_traffic():
    """HBM bytes per launch from the committed hardware-counter summary, if any"""
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(TRAFFIC_FILE).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--variant", default="default", choices=["default", "warmup", "sum", "sum_out", "ternary", "welford", "density"],
                    help="default: Algorithms 2+3; warmup: Theorem 3 warm-up iteration; sum: '(good)' "
                         "update; sum_out: '(good)' update that also writes the int8 vote sums; "
                         "ternary: vote with abstention (tau = 0.05, quorum 2); "
                         "welford / density: the gradient-statistics kernels of Section 3 on one worker's gradient")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target length of the oracle timing")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures one GPU only (the M workers are M buffers on one "
                 "device); run with --gpus 1")

    import torch
    import synth
    import paper_1802_04434_amd as ss

    ss.load_library()            # raises if the HIP library is not built: no fallback
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS[args.workload]
    d, M = cfg.d, cfg.M

    # synthetic inputs of the workload's recipe, generated on the device, untimed
    g = [torch.cat([synth.grad_chunk(cfg, 0, w, c, dev) for c in range(cfg.n_chunks)]) for w in range(M)]
    m = [torch.zeros(d, device=dev) for _ in range(M)] if cfg.beta is not None else None
    x = torch.cat([synth.x0_chunk(cfg, c, dev) for c in range(cfg.n_chunks)])
    voted = ss.new_bits(d, dev)
    beta = cfg.beta if cfg.beta is not None else 0.0
    stream = torch.cuda.current_stream()

    flags = {"default": None, "warmup": ss.STEP_WARMUP, "sum": ss.STEP_SUM_UPDATE,
             "sum_out": ss.STEP_SUM_UPDATE, "ternary": -2, "welford": -1, "density": -1}[args.variant]
    voted_zero = ss.new_bits(d, dev) if args.variant == "ternary" else None
    sums = torch.empty(d, dtype=torch.int8, device=dev) if args.variant == "sum_out" else None
    if args.variant == "welford":
        w_mean, w_m2 = torch.zeros(d, device=dev), torch.zeros(d, device=dev)
    if args.variant == "density":
        phi = torch.zeros(3, dtype=torch.float64, device=dev)
        g32 = g[0].float()

    def step():
        if args.variant == "welford":
            ss.welford_update(g[0], w_mean, w_m2, 7, stream=stream)
        elif args.variant == "density":
            ss.density(g32, phi, stream=stream)
        elif args.variant == "ternary":
            ss.signum_vote_step_ternary(g, m, beta, 0.05, 2, cfg.delta, x, voted, voted_zero, stream=stream)
        elif flags is None:
            ss.signum_vote_step(g, m, beta, cfg.delta, x, voted, None, stream=stream)
        else:
            ss.signum_vote_step_ex(g, m, beta, cfg.delta, x, voted, None, sums, flags, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K launches back to back; wall clock for the job figure, an
    # event pair per launch (same stream) for the kernel figure
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        starts[k].record(stream)
        step()
        stops[k].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    kernel_ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms)

    bytes_per_launch = (algorithmic_bytes_per_coordinate(cfg) + (1 if sums is not None else 0)
                        + (0.125 if args.variant == "ternary" else 0)) * d
    if args.variant == "welford":      # read g, mean, m2; write mean, m2
        bytes_per_launch = ((4 if cfg.grad_dtype == "f32" else 2) + 16) * d
    if args.variant == "density":      # read v
        bytes_per_launch = 4 * d
    achieved = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9

    extra = {"kernel_ms_min": kernel_ms[0], "kernel_ms_median": kernel_ms[len(kernel_ms) // 2],
             "kernel_ms_avg": avg_kernel_ms, "algorithmic_bytes_per_launch": bytes_per_launch}

    if flags == -1:
        name = {"welford": "ss_welford_update", "density": "ss_density (2 launches)"}[args.variant]
        print(json.dumps({
            "metric": "coordinates/sec for %s, d=%d" % (name, d), "value": d / (wall_ms * 1e-3), "unit": "params/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": "%s on one worker's gradient of %s" % (name, cfg.name)},
            "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBS, "traffic": None},
            "cpu_baseline": None, "extra": extra}), flush=True)
        return

    # context: the three-call path (M packs, vote, apply) and a plain copy
    packed = [ss.new_bits(d, dev) for _ in range(M)]
    def three_calls():
        for w in range(M):
            ss.signum_pack(g[w], m[w] if m is not None else None, beta, packed[w], stream=stream)
        ss.majority_vote(packed, voted, d, stream=stream)
        ss.sign_apply(x, voted, cfg.delta, stream=stream)
    for _ in range(3):
        three_calls()
    n3 = max(5, args.steps // 10)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(n3):
        three_calls()
    e1.record(stream)
    torch.cuda.synchronize()
    extra["three_call_path_ms"] = e0.elapsed_time(e1) / n3
    # 1 GiB each way: far beyond the 256 MB memory-side cache, so an HBM figure
    nb = 1 << 30
    src = torch.empty(nb // 4, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        ss.stream_copy(dst, src, nb, stream=stream)
    e0.record(stream)
    for _ in range(20):
        ss.stream_copy(dst, src, nb, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    extra["stream_copy_GBs"] = 2 * nb * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    extra["stream_copy_bytes_each_way"] = nb
    del packed, dst, src

    cpu = None
    if not args.no_cpu_baseline and flags is None:
        cpu = cpu_baseline(cfg, g, args.cpu_seconds)

    out = {
        "metric": "params/sec for fused Signum+vote step (GB/s and %% of HBM peak in roofline), d=%d M=%d" % (d, M),
        "value": d / (wall_ms * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: d=%d %s gradients, M=%d workers, beta=%s, delta=%g, fused ss_signum_vote_step%s"
                               % (cfg.name, d, cfg.grad_dtype, M, cfg.beta, cfg.delta,
                                  "" if flags is None else " variant=" + args.variant)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic() if (args.workload == "C3" and flags is None) else None},
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(out), flush=True)


def cpu_baseline(cfg, g_dev, target_seconds):
    """The CPU oracle, as it stands, on this machine's host cores, same workload."""
    import numpy as np
    import oracle
    import synth

    d, M = cfg.d, cfg.M
    cores = len(os.sched_getaffinity(0))
    # the box advertises its CPU share through OMP_NUM_THREADS
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    g = [synth.as_numpy(t) for t in g_dev]
    m = [np.zeros(d, np.float32) for _ in range(M)] if cfg.beta is not None else None
    x = np.zeros(d, np.float32)
    beta = cfg.beta if cfg.beta is not None else 0.0

    def run(threads):
        t0 = time.perf_counter()
        oracle.signum_vote_step(g, m, beta, cfg.delta, x, threads=threads)
        return time.perf_counter() - t0

    run(cores)                                    # touch every page once
    t_first = run(cores)
    reps = max(1, min(100, int(target_seconds * 0.6 / max(t_first, 1e-6))))
    t_all = sum(run(cores) for _ in range(reps)) / reps
    # one step on a single thread as well, when that stays within a few seconds
    t_one = run(1) if t_first * cores < 0.5 * target_seconds else None
    return {"value": d / t_all, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": "%d full steps of the same workload (d=%d, M=%d) on %d threads, plain C oracle; "
                      "single thread: %s params/s" % (reps, d, M, cores, ("%.4g" % (d / t_one)) if t_one else "not timed"),
            "single_thread_value": (d / t_one) if t_one else None}


if __name__ == "__main__":
    main()
