#!/usr/bin/env python3
"""Benchmark of the Accordion gradient-compression hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic gradients for all W
simulated workers: error-feedback add, gradient accumulation (with the accumulated gradient's
sums of squares), compression at the layer's current level (TopK select + payload + residual, or
the PowerSGD products, orthogonalisation and residual) and the mean over workers.  Every
`window` steps -- max(2, min(--window, steps // 4)), so at least four times at any --steps -- the
per-layer norms are taken and the critical-regime decision picks the next window's levels; every
second window ends with a learning-rate decay, so the levels alternate and both of them, and
the steps right after a switch, are timed.  Gradients are resident in HBM before the timed region
starts (a pool of distinct seeded batches, rotated).

Prints ONE JSON line: gradient GB/s = 4 * N * W / t_step; how many regime tests and steps at each
level the timed region held; the roofline of the dominant kernel (algorithmic bytes / its
HIP-event duration against 8 TB/s; counted HBM traffic from profiles/ if it was taken on the
kernel sources this run uses); the whole step's algorithmic bandwidth; the same figures for the
other target workloads (`other_workloads`); and the CPU oracle's rate on a bounded sample of the
headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")
CSRC = os.path.join(ROOT, "paper_2010_16248_amd", "csrc")


def csrc_digest():
    """Digest of the kernel sources: ties a counter figure in profiles/ to the code it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".h", ".hip")):
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read() + b"\0")
    return h.hexdigest()[:16]


def measured_traffic(workload, W):
    """HBM traffic counted by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, from
    profiles/hbm_traffic_index.txt (one line per workload: workload, W, dominant kernel, its bytes per
    launch, bytes of all kernels of a step, digest of the kernel sources, git commit).  Returns
    (kernel bytes, step bytes, source) -- (None, None, reason) when there is no entry or the kernel
    sources have changed since it was taken: a counter figure of other code is not reported."""
    path = os.path.join(PROFILES, "hbm_traffic_index.txt")
    if not os.path.exists(path):
        return None, None, "no profiles/hbm_traffic_index.txt"
    digest = csrc_digest()
    stale = None
    for line in open(path):
        f = line.split()
        if len(f) < 7 or f[0].startswith("#") or f[0] != workload or int(f[1]) != W:
            continue
        if f[5] != digest:
            stale = f"profiles/hbm_traffic_{workload}.md was taken on other kernel sources (commit {f[6]})"
            continue
        return int(f[3]), int(f[4]), f"profiles/hbm_traffic_{workload}.md at commit {f[6]}"
    return None, None, stale or "workload not profiled"


# Both compression levels are used while timing: the gradient statistics are stationary (every
# window's norm ratio is about 0, i.e. not critical), and every second window ends with a
# learning-rate decay (lr_next < lr_curr), which Algorithm 1 treats as critical.  Decisions:
# critical, not, critical, not, ...
LR_CURR = 0.1


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18_topk",
                    choices=["tiny_powersgd", "resnet18_topk", "resnet18_powersgd", "vgg19_powersgd", "lstm_topk",
                             "resnet18_batch", "resnet18_topk_k99", "lstm_topk_k99"])
    ap.add_argument("--workers", type=int, default=0, help="override W of the workload")
    ap.add_argument("--pool", type=int, default=3, help="distinct gradient batches kept in HBM")
    ap.add_argument("--window", type=int, default=50, help="steps per detection window")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="time only --workload (the default run adds short legs for the other target sets)")
    ap.add_argument("--kernel-events", default="sampled", choices=["sampled", "dominant", "all", "none"],
                    help="which kernels are bracketed with HIP events in the timed region: every fourth "
                         "launch of the fused error-feedback pass (default; a pair of events costs 5-7 us "
                         "of stream time), every launch of it, every kernel, or none")
    ap.add_argument("--fused-update", action="store_true",
                    help="end every step with the fused Nesterov-momentum update of weights and velocity "
                         "(accordion_step_all_update) instead of storing the averaged gradient")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture one step per pool batch in a HIP graph (torch.cuda.CUDAGraph) and replay "
                         "it; per-kernel events are off then")
    ap.add_argument("--fixed-level", type=int, default=-1, help="0/1: never switch, use this level")
    ap.add_argument("--probe-mib", type=int, default=1024,
                    help="size of the plain-copy probe (MiB read and MiB written per launch); 0: skip")
    return ap.parse_args()


def dominant_kernel(method):
    from paper_2010_16248_amd import binding as B
    if method == B.ACC_BATCH:
        return "batch_micro_kernel"
    return "topk_ef_hist_kernel" if method == B.ACC_TOPK else "psgd_ef_p_kernel"


def algorithmic_bytes_dominant(n_params, W):
    """Fused error-feedback pass: per worker read g and e, write Delta (12 B / element); worker 0
    also reads and writes the accumulator (8 B / element)."""
    return n_params * (12 * W + 8)


def algorithmic_bytes_batch(n_model, W, micro_steps, exchanges):
    """Batch-size mode, total over `micro_steps` launches that completed `exchanges` batches: every
    micro-step reads W gradients and reads and writes the accumulator; a batch of n micro-steps
    writes and re-reads the W running sums n - 1 times; every completed batch writes D."""
    return n_model * ((4 * W + 8) * micro_steps + 8 * W * (micro_steps - exchanges) + 4 * exchanges)


def algorithmic_bytes_step(w, layers, W, levels_k_or_r):
    """Bytes the method itself must move per step (one read/write of each operand per pass)."""
    from paper_2010_16248_amd import binding as B
    N = sum(l.numel for l in layers)
    if w.method == B.ACC_TOPK:
        kept = sum(levels_k_or_r)
        return 12 * N * W + 8 * N + 8 * kept * W + 4 * N
    mat = sum(l.numel for l in layers if l.is_matrix)
    vec = N - mat
    return 24 * mat * W + 8 * N + 4 * N + 4 * vec * W


def cpu_baseline(w, W, n_steps, window):
    """The oracle as it stands, single BLAS thread, on the same seeded inputs."""
    from oracle import accordion_oracle as orc
    from paper_2010_16248_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    layers = [(l.offset, l.rows, l.cols, l.is_matrix) for l in w.layers]
    if w.method == 2:
        return cpu_baseline_batch(w, W, layers, orc, wl, threadpool_limits)
    rmax = max(w.level_crit, w.level_noncrit)
    q0 = wl.q_init(w, rmax, w.seed) if w.method == 0 else None
    ora = orc.AccordionOracle(w.method, layers, W, w.level_crit, w.level_noncrit, w.k_den, w.eta, 1, q0)
    # a bounded sample: whole steps until about 12 s of oracle time have passed (one step at
    # least, n_steps at most); the inputs are generated outside the timed parts
    ctx = threadpool_limits(limits=1) if threadpool_limits else None
    spent, done = 0.0, 0
    while done < n_steps and (done == 0 or spent < 12.0):
        g = [wl.gradient(w, k, done) for k in range(W)]
        t0 = time.perf_counter()
        ora.step(g)
        spent += time.perf_counter() - t0
        done += 1
    t0 = time.perf_counter()
    ora.detect_regime(0.1, 0.1)          # one window end
    spent += time.perf_counter() - t0
    if ctx is not None:
        ctx.restore_original_limits()
    n_steps = done
    per_step = spent / n_steps
    gbs = 4.0 * w.n_params * W / per_step / 1e9
    return {"value": round(gbs, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_steps} full steps of {w.name} (all {W} workers, every layer) + 1 regime test, "
                      f"numpy oracle, 1 thread, {per_step:.3f} s/step",
            "host_cpus": os.cpu_count()}


def cpu_baseline_batch(w, W, layers, orc, wl, threadpool_limits):
    """Batch-size mode: one full large batch (multiplier micro-steps) + one whole-model test."""
    ora = orc.BatchSizeOracle(layers, W, w.batch_multiplier, w.eta, 0, True)
    n_steps = w.batch_multiplier
    grads = [[wl.gradient(w, k, s % 3) for k in range(W)] for s in range(n_steps)]
    ctx = threadpool_limits(limits=1) if threadpool_limits else None
    t0 = time.perf_counter()
    for s in range(n_steps):
        ora.micro_step(grads[s])
    ora.detect_regime(0.1, 0.1)
    t1 = time.perf_counter()
    if ctx is not None:
        ctx.restore_original_limits()
    per_step = (t1 - t0) / n_steps
    return {"value": round(4.0 * w.n_params * W / per_step / 1e9, 4), "unit": "GB/s", "cores": 1,
            "kind": "oracle",
            "sample": f"{n_steps} micro-steps (one large batch) of {w.name}, all {W} workers + 1 whole-model "
                      f"regime test, numpy oracle, 1 thread, {per_step:.3f} s/micro-step",
            "host_cpus": os.cpu_count()}


def window_steps(args, steps):
    """Detection window used while timing: at most --window, and short enough that the timed steps
    hold at least four window ends (two with a learning-rate decay, two without)."""
    return max(2, min(args.window, steps // 4))


def make_gradient_pool(w, W, pool, dev, wl):
    """pool x W seeded gradients, resident in HBM.  Generated on the host by the shared seeded
    module (several at a time: the large sets take seconds each)."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    jobs = [(s, k) for s in range(pool) for k in range(W)]
    threads = min(8, len(jobs)) if w.n_params > 30_000_000 else 1
    out = [[None] * W for _ in range(pool)]
    if threads > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            for (s, k), g in zip(jobs, ex.map(lambda sk: wl.gradient(w, sk[1], sk[0]), jobs)):
                out[s][k] = torch.from_numpy(g).to(dev)
    else:
        for s, k in jobs:
            out[s][k] = torch.from_numpy(wl.gradient(w, k, s)).to(dev)
    return out


def measure(name, args, steps, warmup, pool, full):
    """Time `steps` whole steps of one workload.  full: the primary workload of the run (options
    of the command line apply, copy probe, per-kernel table); else a short leg with defaults."""
    import torch
    from paper_2010_16248_amd import binding as B
    from paper_2010_16248_amd import workloads as wl

    w = wl.workload(name)
    W = args.workers if (full and args.workers > 0) else w.n_workers
    layers = w.layers
    N = w.n_params
    rmax = max(w.level_crit, w.level_noncrit)
    q0 = wl.q_init(w, rmax, w.seed) if w.method == B.ACC_POWERSGD else None
    is_batch = w.method == B.ACC_BATCH
    fused = full and args.fused_update
    fixed_level = args.fixed_level if full else -1
    hip_graph = full and args.hip_graph
    kernel_events = args.kernel_events if full else "sampled"
    gpu = B.Accordion(w.method, layers, W, w.level_crit, w.level_noncrit, w.k_den, w.eta, 1, q0,
                      batch_multiplier=w.batch_multiplier)

    dev = torch.device("cuda:0")
    base = make_gradient_pool(w, W, pool, dev, wl)
    out = torch.empty(N, dtype=torch.float32, device=dev)
    weights = velocity = None
    if fused:
        weights = torch.full((N,), 0.01, dtype=torch.float32, device=dev)
        velocity = torch.zeros(N, dtype=torch.float32, device=dev)
    if fixed_level in (0, 1):
        st = gpu.unpack_state(gpu.get_state())
        blob = gpu.pack_state(st["e"], st["A"], st["Q"], st["norm_old"], st["has_old"],
                              np.full(gpu.n_layers, fixed_level, np.int32), 0)
        gpu.set_state(blob)

    # plain copy of known size: the copy bandwidth this machine reaches, and the kernel that calibrates
    # FETCH_SIZE / WRITE_SIZE in a rocprofv3 --pmc run of this file
    copy_probe = None
    if full and args.probe_mib > 0:
        n = args.probe_mib * (1 << 20) // 4
        src = torch.full((n,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            B.probe_copy(dst, src)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        ev0.record()
        for _ in range(reps):
            B.probe_copy(dst, src)
        ev1.record()
        torch.cuda.synchronize()
        us = ev0.elapsed_time(ev1) * 1e3 / reps
        copy_probe = {"bytes_read": 4 * n, "bytes_written": 4 * n, "avg_us": round(us, 2),
                      "GB/s": round(8.0 * n / us / 1e3, 1)}
        del src, dst

    window = window_steps(args, steps)
    state = {"step": 0, "tests": 0, "decays": 0}
    graphs = None
    if hip_graph:
        kernel_events = "none"
        if is_batch and pool % 2:
            print("bench.py: --hip-graph in batch-size mode needs an even --pool", file=sys.stderr)
            sys.exit(2)

    def one_step():
        s = state["step"]
        if graphs is not None:
            graphs[s % pool].replay()
        elif fused:
            gpu.step_all_update(base[s % pool], weights, velocity, LR_CURR, 0.9, 0.0)
        else:
            gpu.step_all(base[s % pool], out)
        if fixed_level < 0 and (s + 1) % window == 0:
            # every second window ends with an LR decay (not in batch-size mode, where the large
            # batch, once reached, is kept: the timed region is the steady state)
            decay = ((s + 1) // window) % 2 == 1 and not is_batch
            gpu.detect_regime(LR_CURR, LR_CURR * 0.1 if decay else LR_CURR)
            state["tests"] += 1
            state["decays"] += 1 if decay else 0
        state["step"] = s + 1

    # the warm-up runs whole windows, so that the timed region starts at a window boundary with the
    # level the last (decay-free) window end chose
    for _ in range(-(-max(warmup, 1) // (2 * window)) * 2 * window if fixed_level < 0 else warmup):
        one_step()
    torch.cuda.synchronize()
    if hip_graph:
        # steady state reached: capture one step per pool batch on a side stream
        side = torch.cuda.Stream()
        gpu.set_stream(side.cuda_stream)
        captured = []
        for b in range(pool):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                if fused:
                    gpu.step_all_update(base[b], weights, velocity, LR_CURR, 0.9, 0.0)
                else:
                    gpu.step_all(base[b], out)
            captured.append(g)
        graphs = captured
        torch.cuda.synchronize()
        gpu.set_stream(torch.cuda.current_stream().cuda_stream)   # replays and eager calls share a stream
    state.update(step=0, tests=0, decays=0)    # the timed region starts at a window boundary
    use_events = kernel_events != "none"
    if use_events:
        gpu.set_profiling({"all": 1, "dominant": 2, "sampled": 3}[kernel_events])
    words0 = gpu.payload_words()[1]
    stats0 = gpu.topk_stats() if w.method == B.ACC_TOPK else None
    torch.cuda.synchronize()
    bs0 = gpu.batch_status() if is_batch else None
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
    gpu.flush()                            # the last step's residual is written out
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = gpu.get_profile() if use_events else {}
    if use_events:
        gpu.set_profiling(False)
    ms_per_step = (t1 - t0) * 1e3 / steps
    value = 4.0 * N * W / (ms_per_step * 1e-3) / 1e9

    levels = gpu.get_levels()
    words_last, words_cum = gpu.payload_words()

    # how many of the timed steps ran at which level: from the floats sent (every layer switches
    # with the others here, so a step sends the critical or the non-critical amount)
    steps_crit = steps_noncrit = None
    if not is_batch:
        lt = [(l.offset, l.rows, l.cols, l.is_matrix) for l in layers]
        wc = payload_words_at(w, lt, 1)
        wn = payload_words_at(w, lt, 0)
        sent = words_cum - words0
        if fixed_level in (0, 1):
            steps_crit, steps_noncrit = (steps, 0) if fixed_level == 1 else (0, steps)
        elif wc != wn:
            steps_crit = (sent - steps * wn) / (wc - wn)
            steps_noncrit = steps - steps_crit
            if abs(steps_crit - round(steps_crit)) < 1e-9:
                steps_crit, steps_noncrit = int(round(steps_crit)), int(round(steps_noncrit))

    dom = dominant_kernel(w.method)
    roofline = None
    kernels = {}
    k_traffic, step_traffic, traffic_src = measured_traffic(name, W)
    if prof:
        tot = sum(ms for ms, _ in prof.values())
        for kname, (ms, n) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            kernels[kname] = {"avg_us": round(ms * 1e3 / n, 2), "launches": n, "share": round(ms / tot, 3)}
        if is_batch and fused:
            dom = "batch_micro_update_kernel"
        ms, n = prof[dom]
        avg_s = ms * 1e-3 / n
        if is_batch:
            bs1 = gpu.batch_status()
            steps_t, exch_t = bs1["micro_steps"] - bs0["micro_steps"], bs1["exchanges"] - bs0["exchanges"]
            alg_bytes = algorithmic_bytes_batch(N, W, steps_t, exch_t) // max(1, steps_t)
            if fused:
                alg_bytes += 12 * N * exch_t // max(1, steps_t)     # w, v read and written, no D store
        else:
            alg_bytes = algorithmic_bytes_dominant(N, W)
        ach = alg_bytes / avg_s / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": k_traffic,
                    "traffic_source": traffic_src,
                    "avg_kernel_us": round(avg_s * 1e6, 2), "launches_timed": n,
                    "algorithmic_bytes_per_launch": alg_bytes}

    # the whole step: bytes the method must move (one read / write of each operand per pass, the
    # payload at the levels the timed steps ran at) and the traffic counted by rocprofv3 for all kernels
    step_bw = None
    if not is_batch:
        kept = (sent // 2) / steps if w.method == B.ACC_TOPK else 0
        alg = algorithmic_bytes_step(w, layers, W, [kept])
        cnt = step_traffic
        if fused:                            # weights and velocity read and written instead of D written
            alg += 12 * N
            cnt = None                       # counted for the storing sink only
        t_s = ms_per_step * 1e-3
        step_bw = {"algorithmic_bytes": int(alg), "algorithmic_GB/s": round(alg / t_s / 1e9, 1),
                   "algorithmic_frac_of_peak": round(alg / t_s / 1e9 / HBM_PEAK_GBS, 4),
                   "counted_bytes": cnt, "counted_source": traffic_src,
                   "counted_GB/s": round(cnt / t_s / 1e9, 1) if cnt else None,
                   "counted_frac_of_peak": round(cnt / t_s / 1e9 / HBM_PEAK_GBS, 4) if cnt else None}

    res = {
        "value": round(value, 2), "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": name, "n_params": N, "n_workers": W, "n_layers": len(layers),
                   "method": {B.ACC_TOPK: "topk", B.ACC_POWERSGD: "powersgd", B.ACC_BATCH: "batch"}[w.method],
                   "batch_multiplier": w.batch_multiplier,
                   "level_crit": w.level_crit, "level_noncrit": w.level_noncrit,
                   "window_steps": window, "pool_batches": pool,
                   "regime_tests_in_timed_region": state["tests"],
                   "of_which_with_lr_decay": state["decays"],
                   "steps_at_crit": steps_crit, "steps_at_noncrit": steps_noncrit,
                   "hip_graph": bool(hip_graph),
                   "sink": "nesterov update of weights and velocity" if fused else "averaged gradient stored",
                   "kernel_events_in_timed_region": kernel_events},
        "roofline": roofline, "step_bandwidth": step_bw, "copy_probe": copy_probe, "kernels": kernels,
        "payload_words_last_step": words_last, "critical_layers_at_end": int(levels.sum()),
    }
    if stats0 is not None:
        s1 = gpu.topk_stats()
        res["topk_paths"] = {"layer_steps": steps * W * len(layers), "guess_missed": s1[0] - stats0[0],
                             "tie_sweeps": s1[1] - stats0[1]}
    gpu.destroy()
    del base, out
    torch.cuda.empty_cache()
    return res, w, W


def payload_words_at(w, layer_tuples, level):
    """Floats one worker sends per step when every layer is at `level` (the paper's accounting)."""
    val = w.level_crit if level == 1 else w.level_noncrit
    total = 0
    for (_, rows, cols, is_m) in layer_tuples:
        n = rows * cols
        if w.method == 0:
            total += max(1, min(val, rows, cols)) * (rows + cols) if is_m else n
        else:
            total += 2 * max(1, -((-n * val) // w.k_den))
    return total


OTHER_WORKLOADS = ["resnet18_powersgd", "vgg19_powersgd", "lstm_topk"]


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "the path would shard by worker (one data-parallel worker per GPU)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2010_16248_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load_library()                       # fails loudly if the HIP library is missing
    res, w, W = measure(args.workload, args, args.steps, args.warmup, args.pool, True)

    # the other target sets, timed the same way in short legs (no per-kernel table, no CPU leg)
    others = []
    if not args.no_other_workloads:
        for name in OTHER_WORKLOADS:
            if name == args.workload:
                continue
            o_steps = max(args.steps, 40)
            o, _, oW = measure(name, args, o_steps, max(args.warmup, 10), 2 if name.startswith("lstm") else 3, False)
            rf, sb = o["roofline"] or {}, o["step_bandwidth"] or {}
            others.append({"workload": name, "n_workers": oW, "steps": o_steps, "ms_per_step": o["ms_per_step"],
                           "gradient_GB/s": o["value"],
                           "dominant_kernel": rf.get("kernel"), "dominant_kernel_us": rf.get("avg_kernel_us"),
                           "dominant_kernel_frac_of_peak": rf.get("frac"),
                           "step_algorithmic_frac_of_peak": sb.get("algorithmic_frac_of_peak"),
                           "step_counted_frac_of_peak": sb.get("counted_frac_of_peak"),
                           "regime_tests_in_timed_region": o["config"]["regime_tests_in_timed_region"],
                           "steps_at_crit": o["config"]["steps_at_crit"],
                           "steps_at_noncrit": o["config"]["steps_at_noncrit"],
                           "topk_paths": o.get("topk_paths")})

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, W, 400, args.window)

    line = {
        "metric": "gradient GB/s per compress step (EF+compress+norm)",
        "value": res["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": res["config"],
        "roofline": res["roofline"],
        "step_bandwidth": res["step_bandwidth"],
        "cpu_baseline": cpu,
        "copy_probe": res["copy_probe"],
        "kernels": res["kernels"],
        "payload_words_last_step": res["payload_words_last_step"],
        "critical_layers_at_end": res["critical_layers_at_end"],
        "topk_paths": res.get("topk_paths"),
        "other_workloads": others,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
