#!/usr/bin/env python3
"""Benchmark of the signSGD / Signum majority-vote hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--kernel fused]

A step is one pass of the whole hot path over one batch of synthetic
gradients that already sit in HBM: by default one ss_signum_vote_step call over
all M workers (momentum, sign, vote, parameter update in one kernel).  The
headline workload is C3: d = 25,557,032 fp32 parameters, M = 7, beta = 0.9.

Prints ONE JSON line: params/s, the HBM roofline of the kernel (algorithmic
bytes per launch / mean launch duration from HIP events on the launch's own
stream, against 8 TB/s) and the CPU oracle timed on this machine's host cores.

--kernel selects what a "step" is.  Besides `fused` there are the variants of
the step (warmup, sum, sum_out, ternary) and every stand-alone entry point of
the library (pack, vote, apply, three_calls, vote_sum, sum_apply, pack_ternary,
quorum_vote, ternary_apply, welford, welford_sigma, density), each on buffers of
the chosen workload, each with its own algorithmic byte count and the matching
oracle routine as CPU baseline.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def library_source_digest():
    """sha256 over the kernel sources and the header: names the code a profile was taken with"""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_1802_04434_amd", "csrc")
    files = sorted(os.path.join(src, f) for f in os.listdir(src) if f.endswith((".hip", ".hpp")))
    for f in files + [os.path.join(ROOT, "include", "signsgd.h")]:
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def counter_traffic(workload):
    """HBM bytes per launch of the fused step from the committed hardware-counter
    summary of that workload (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the copy
    kernel) - but only if the summary was taken with exactly the sources this run
    uses (it records their digest); otherwise None."""
    try:
        text = open(os.path.join(ROOT, "profiles", "fused_step_%s_profile.md" % workload)).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    s = re.search(r"library_source_digest:\s*([0-9a-f]+)", text)
    if not m or not s or s.group(1) != library_source_digest():
        return None
    return float(m.group(1))


def bytes_per_coordinate(kernel, cfg):
    """What the method itself must move per coordinate and launch."""
    M = cfg.M
    gb = 4 if cfg.grad_dtype == "f32" else 2
    mom = 8 if cfg.beta is not None else 0          # read m, write m
    fused = M * (gb + mom) + 8 + 0.125              # every worker's g (and m), x in and out, one voted bit
    return {
        "fused": fused, "warmup": fused, "sum": fused, "sum_out": fused + 1,
        "ternary": fused + 0.125,                   # two voted planes
        "pack": gb + mom + 0.125,                   # one worker: g (and m), its bits
        "vote": (M + 1) / 8.0,
        "apply": 8.125,
        "three_calls": M * (gb + mom + 0.25) + 8.25,
        "vote_sum": M / 8.0 + 1,                    # M packed words in, one int8 out
        "sum_apply": 9.0,                           # x in and out, one int8
        "pack_ternary": gb + mom + 0.25,            # one worker: g (and m), two planes
        "quorum_vote": (2 * M + 2) / 8.0,
        "ternary_apply": 8.25,
        "welford": gb + 16,                         # g, mean and m2 in; mean and m2 out
        "welford_sigma": 8.0,
        "density": 4.0,
    }[kernel]


KERNELS = ["fused", "warmup", "sum", "sum_out", "ternary", "pack", "vote", "apply", "three_calls", "vote_sum",
           "sum_apply", "pack_ternary", "quorum_vote", "ternary_apply", "welford", "welford_sigma", "density"]
ENTRY_POINT = {
    "fused": "ss_signum_vote_step", "warmup": "ss_signum_vote_step_ex(SS_STEP_WARMUP)",
    "sum": "ss_signum_vote_step_ex(SS_STEP_SUM_UPDATE)", "sum_out": "ss_signum_vote_step_ex(SS_STEP_SUM_UPDATE, sums_out)",
    "ternary": "ss_signum_vote_step_ternary(tau=0.05, quorum=2)", "pack": "ss_signum_pack (worker 0)",
    "vote": "ss_majority_vote", "apply": "ss_sign_apply", "three_calls": "M x ss_signum_pack + ss_majority_vote + ss_sign_apply",
    "vote_sum": "ss_vote_sum", "sum_apply": "ss_sum_apply", "pack_ternary": "ss_signum_pack_ternary (worker 0, tau=0.05)",
    "quorum_vote": "ss_quorum_vote(quorum=2)", "ternary_apply": "ss_ternary_apply", "welford": "ss_welford_update (worker 0)",
    "welford_sigma": "ss_welford_sigma", "density": "ss_density (worker 0's gradient as fp32)",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--kernel", "--variant", dest="kernel", default="fused", choices=KERNELS + ["default"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true", help="skip the three-call / copy / graph context figures")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target length of the oracle timing")
    args = ap.parse_args()
    if args.kernel == "default":
        args.kernel = "fused"
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
    d, M, kernel = cfg.d, cfg.M, args.kernel
    has_m = cfg.beta is not None
    beta = cfg.beta if has_m else 0.0
    tau, quorum = 0.05, 2

    # synthetic inputs of the workload's recipe, generated on the device, untimed
    g = [torch.cat([synth.grad_chunk(cfg, 0, w, c, dev) for c in range(cfg.n_chunks)]) for w in range(M)]
    m = [torch.zeros(d, device=dev) for _ in range(M)] if has_m else None
    x = torch.cat([synth.x0_chunk(cfg, c, dev) for c in range(cfg.n_chunks)])
    voted = ss.new_bits(d, dev)
    stream = torch.cuda.current_stream()     # the library's launches and the timing events share it

    # buffers that only some kernels need
    need_packed = kernel in ("vote", "apply", "three_calls", "vote_sum")
    packed = [ss.new_bits(d, dev) for _ in range(M)] if need_packed else None
    if need_packed:
        for w in range(M):
            ss.signum_pack(g[w], None, 0.0, packed[w], stream=stream)
    if kernel in ("ternary", "quorum_vote", "ternary_apply"):
        voted_zero = ss.new_bits(d, dev)
    if kernel in ("quorum_vote", "ternary_apply", "pack_ternary"):
        neg = [ss.new_bits(d, dev) for _ in range(M if kernel != "pack_ternary" else 1)]
        zero = [ss.new_bits(d, dev) for _ in range(len(neg))]
        for w in range(len(neg)):
            ss.signum_pack_ternary(g[w], None, 0.0, tau, neg[w], zero[w], stream=stream)
    if kernel in ("sum_out", "vote_sum", "sum_apply"):
        sums = torch.zeros(d, dtype=torch.int8, device=dev)
        if kernel == "sum_apply":
            tmp = [ss.new_bits(d, dev) for _ in range(M)]
            for w in range(M):
                ss.signum_pack(g[w], None, 0.0, tmp[w], stream=stream)
            ss.vote_sum(tmp, sums, d, stream=stream)
            del tmp
    if kernel in ("welford", "welford_sigma"):
        w_mean, w_m2 = torch.zeros(d, device=dev), torch.rand(d, device=dev)
        sigma = torch.empty(d, device=dev)
    if kernel == "density":
        phi = torch.zeros(3, dtype=torch.float64, device=dev)
        work = ss.new_density_workspace(dev)
        g32 = g[0].float()
    if kernel in ("apply", "ternary_apply"):
        ss.majority_vote(packed, voted, d, stream=stream) if kernel == "apply" else \
            ss.quorum_vote(neg, zero, quorum, voted, voted_zero, d, stream=stream)

    def step():
        if kernel == "fused":
            ss.signum_vote_step(g, m, beta, cfg.delta, x, voted, None, stream=stream)
        elif kernel == "warmup":
            ss.signum_vote_step_ex(g, m, beta, cfg.delta, x, voted, None, None, ss.STEP_WARMUP, stream=stream)
        elif kernel == "sum":
            ss.signum_vote_step_ex(g, m, beta, cfg.delta, x, voted, None, None, ss.STEP_SUM_UPDATE, stream=stream)
        elif kernel == "sum_out":
            ss.signum_vote_step_ex(g, m, beta, cfg.delta, x, voted, None, sums, ss.STEP_SUM_UPDATE, stream=stream)
        elif kernel == "ternary":
            ss.signum_vote_step_ternary(g, m, beta, tau, quorum, cfg.delta, x, voted, voted_zero, stream=stream)
        elif kernel == "pack":
            ss.signum_pack(g[0], m[0] if has_m else None, beta, voted, stream=stream)
        elif kernel == "vote":
            ss.majority_vote(packed, voted, d, stream=stream)
        elif kernel == "apply":
            ss.sign_apply(x, voted, cfg.delta, stream=stream)
        elif kernel == "three_calls":
            for w in range(M):
                ss.signum_pack(g[w], m[w] if has_m else None, beta, packed[w], stream=stream)
            ss.majority_vote(packed, voted, d, stream=stream)
            ss.sign_apply(x, voted, cfg.delta, stream=stream)
        elif kernel == "vote_sum":
            ss.vote_sum(packed, sums, d, stream=stream)
        elif kernel == "sum_apply":
            ss.sum_apply(x, sums, cfg.delta, stream=stream)
        elif kernel == "pack_ternary":
            ss.signum_pack_ternary(g[0], m[0] if has_m else None, beta, tau, neg[0], zero[0], stream=stream)
        elif kernel == "quorum_vote":
            ss.quorum_vote(neg, zero, quorum, voted, voted_zero, d, stream=stream)
        elif kernel == "ternary_apply":
            ss.ternary_apply(x, voted, voted_zero, cfg.delta, stream=stream)
        elif kernel == "welford":
            ss.welford_update(g[0], w_mean, w_m2, 7, stream=stream)
        elif kernel == "welford_sigma":
            ss.welford_sigma(w_m2, 7, sigma, stream=stream)
        elif kernel == "density":
            ss.density(g32, phi, work, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps back to back.  Wall clock (with a synchronize on both sides) gives the
    # job figure; one HIP event pair around the K launches, on the stream they run on, gives the
    # mean launch duration (the launches queue up behind each other, so host launch overhead is
    # hidden as it is in a training loop).
    e_begin, e_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e_begin.record(stream)
    for k in range(args.steps):
        step()
    e_end.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    avg_kernel_ms = e_begin.elapsed_time(e_end) / args.steps
    # spread of single launches, each between its own event pair (adds a few us per launch)
    n_single = min(args.steps, 50)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(n_single)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(n_single)]
    for k in range(n_single):
        starts[k].record(stream)
        step()
        stops[k].record(stream)
    torch.cuda.synchronize()
    kernel_ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))

    bytes_per_launch = bytes_per_coordinate(kernel, cfg) * d
    achieved = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    extra = {"kernel_ms_avg": avg_kernel_ms, "single_launch_ms_min": kernel_ms[0],
             "single_launch_ms_median": kernel_ms[len(kernel_ms) // 2],
             "algorithmic_bytes_per_launch": bytes_per_launch,
             "algorithmic_bytes_per_coordinate": bytes_per_coordinate(kernel, cfg),
             "library_source_digest": library_source_digest()}
    if bytes_per_launch < 256e6:
        extra["note"] = ("%.0f MB per launch fit the 256 MB memory-side cache and take %.1f us at HBM peak: "
                         "launch / latency bound, not an HBM figure" % (bytes_per_launch / 1e6, bytes_per_launch / 8e6))

    if kernel == "fused" and not args.no_context:
        context_figures(ss, torch, cfg, g, m, x, voted, beta, stream, dev, args, extra, step)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(kernel, cfg, g, args.cpu_seconds, tau, quorum)

    out = {
        "metric": "params/sec for %s (GB/s and %% of HBM peak in roofline), d=%d M=%d" % (
            "fused Signum+vote step" if kernel == "fused" else ENTRY_POINT[kernel], d, M),
        "value": d / (wall_ms * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.grad_dtype if cfg.grad_dtype == "f32" else "bf16 gradients, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": "%s: d=%d %s gradients, M=%d workers, beta=%s, delta=%g, %s"
                               % (cfg.name, d, cfg.grad_dtype, M, cfg.beta, cfg.delta, ENTRY_POINT[kernel])},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": counter_traffic(args.workload) if kernel == "fused" else None},
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(out), flush=True)


def context_figures(ss, torch, cfg, g, m, x, voted, beta, stream, dev, args, extra, step):
    """Around the headline number: the same step as M + 2 calls, a plain copy,
    and - where a launch is a few microseconds - the step replayed from a HIP graph."""
    d, M = cfg.d, cfg.M
    has_m = m is not None
    packed = [ss.new_bits(d, dev) for _ in range(M)]

    def three_calls():
        for w in range(M):
            ss.signum_pack(g[w], m[w] if has_m else None, beta, packed[w], stream=stream)
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
    del packed
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
    del dst, src
    if cfg.d < (1 << 22):
        # launch bound: K steps captured once in a HIP graph and replayed, against K eager launches
        K = 20
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(K):
                    ss.signum_vote_step(g, m, beta, cfg.delta, x, voted, None, stream=side)
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            graph.replay()
        torch.cuda.synchronize()
        extra["graph_replay_us_per_step"] = (time.perf_counter() - t0) * 1e6 / (20 * K)
        e0.record(stream)
        for _ in range(20 * K):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        extra["eager_back_to_back_us_per_step"] = e0.elapsed_time(e1) * 1e3 / (20 * K)


def cpu_baseline(kernel, cfg, g_dev, target_seconds, tau, quorum):
    """The CPU oracle as it stands, on this machine's host cores, on a bounded sample of
    the same workload.  The fused step uses the oracle's threaded entry point on the
    full vector; every other routine is single-threaded in the oracle and is timed on
    a leading slice of the vector."""
    import numpy as np
    import oracle
    import synth

    d, M = cfg.d, cfg.M
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))   # the box advertises its CPU share there
    has_m = cfg.beta is not None
    beta = cfg.beta if has_m else 0.0

    if kernel == "fused":
        n = min(d, 1 << 27)                      # at most 2^27 coordinates resident on the host
        g = [synth.as_numpy(t[:n]) for t in g_dev]
        m = [np.zeros(n, np.float32) for _ in range(M)] if has_m else None
        x = np.zeros(n, np.float32)

        def run(threads):
            t0 = time.perf_counter()
            oracle.signum_vote_step(g, m, beta, cfg.delta, x, threads=threads)
            return time.perf_counter() - t0
        run(cores)                                    # touch every page once
        t_first = run(cores)
        reps = max(1, min(100, int(target_seconds * 0.6 / max(t_first, 1e-6))))
        t_all = sum(run(cores) for _ in range(reps)) / reps
        t_one = run(1) if t_first * cores < 0.5 * target_seconds else None
        return {"value": n / t_all, "unit": "params/s", "cores": cores, "kind": "oracle",
                "sample": "%d steps over the first %d of %d coordinates (M=%d) on %d threads, plain C oracle "
                          "(sso_signum_vote_step_mt); single thread: %s params/s"
                          % (reps, n, d, M, cores, ("%.4g" % (n / t_one)) if t_one else "not timed"),
                "single_thread_value": (n / t_one) if t_one else None}

    # single-threaded oracle routines on a slice
    n = min(d, 1 << 22)
    g = [synth.as_numpy(t[:n]) for t in g_dev]
    m = [np.zeros(n, np.float32) for _ in range(M)] if has_m else None
    x = np.zeros(n, np.float32)
    packed = [oracle.signum_pack(a, None, 0.0) for a in g]
    voted = oracle.majority_vote(packed, n)
    tern = [oracle.signum_pack_ternary(a, None, 0.0, tau) for a in g]
    negs, zeros = [t[0] for t in tern], [t[1] for t in tern]
    vneg, vzero = oracle.quorum_vote(negs, zeros, quorum, n)
    sums = oracle.vote_sum(packed, n).astype(np.int8)
    mean, m2 = np.zeros(n, np.float32), np.ones(n, np.float32)
    g32 = g[0] if g[0].dtype == np.float32 else (g[0].astype(np.uint32) << 16).view(np.float32)
    flags = {"warmup": oracle.STEP_WARMUP, "sum": oracle.STEP_SUM_UPDATE, "sum_out": oracle.STEP_SUM_UPDATE}
    calls = {
        "warmup": lambda: oracle.signum_vote_step_ex(g, m, beta, cfg.delta, x, flags["warmup"]),
        "sum": lambda: oracle.signum_vote_step_ex(g, m, beta, cfg.delta, x, flags["sum"]),
        "sum_out": lambda: oracle.signum_vote_step_ex(g, m, beta, cfg.delta, x, flags["sum_out"]),
        "ternary": lambda: oracle.signum_vote_step_ternary(g, m, beta, tau, quorum, cfg.delta, x),
        "pack": lambda: oracle.signum_pack(g[0], m[0] if has_m else None, beta),
        "vote": lambda: oracle.majority_vote(packed, n),
        "apply": lambda: oracle.sign_apply(x, voted, cfg.delta),
        "three_calls": lambda: (
            [oracle.signum_pack(g[w], m[w] if has_m else None, beta) for w in range(M)],
            oracle.majority_vote(packed, n), oracle.sign_apply(x, voted, cfg.delta)),
        "vote_sum": lambda: oracle.vote_sum(packed, n),
        "sum_apply": lambda: oracle.sum_apply(x, sums, cfg.delta),
        "pack_ternary": lambda: oracle.signum_pack_ternary(g[0], m[0] if has_m else None, beta, tau),
        "quorum_vote": lambda: oracle.quorum_vote(negs, zeros, quorum, n),
        "ternary_apply": lambda: oracle.ternary_apply(x, vneg, vzero, cfg.delta),
        "welford": lambda: oracle.welford_update(g[0], mean, m2, 7),
        "welford_sigma": lambda: oracle.welford_sigma(m2, 7),
        "density": lambda: oracle.density(g32),
    }
    call = calls[kernel]
    call()
    t0 = time.perf_counter()
    call()
    t_first = time.perf_counter() - t0
    reps = max(1, min(200, int(0.5 * target_seconds / max(t_first, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(reps):
        call()
    t_all = (time.perf_counter() - t0) / reps
    return {"value": n / t_all, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": "%d calls of the matching single-threaded oracle routine on the first %d of %d coordinates (M=%d)"
                      % (reps, n, d, M), "single_thread_value": n / t_all}


if __name__ == "__main__":
    main()
