#!/usr/bin/env python3
"""Benchmark of the Accordion gradient-compression hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic gradients for all W
simulated workers: error-feedback add, gradient accumulation, compression at the layer's current
level (TopK select + payload + residual, or the PowerSGD products, orthogonalisation and
residual), the mean over workers, and -- every `window` steps -- the per-layer norms and the
critical-regime decision that picks the next window's levels.  Gradients are resident in HBM
before the timed region starts (a pool of distinct seeded batches, rotated).

Prints ONE JSON line: gradient GB/s = 4 * N * W / t_step, plus the roofline of the dominant
kernel (algorithmic bytes / its HIP-event duration against 8 TB/s) and the CPU oracle's rate on
a bounded sample of the same workload.
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

# HBM traffic of the dominant kernel per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# of this file (summaries under profiles/); None until measured for a workload.
# Key: (workload, W, dominant kernel).
MEASURED_TRAFFIC_BYTES = {
    ("resnet18_topk", 4, "topk_ef_hist_kernel"): 657244796,      # profiles/hbm_traffic_resnet18_topk.md
    ("resnet18_powersgd", 4, "psgd_ef_p_kernel"): 635250034,     # profiles/hbm_traffic_resnet18_powersgd.md
    ("vgg19_powersgd", 1, "psgd_ef_p_kernel"): 416681243,        # profiles/hbm_traffic_vgg19_powersgd.md
    ("lstm_topk", 16, "topk_ef_hist_kernel"): 10615536735,       # profiles/hbm_traffic_lstm_topk.md
    ("resnet18_topk_k99", 4, "topk_ef_hist_kernel"): 637193697,  # profiles/hbm_traffic_resnet18_topk_k99.md
    ("resnet18_batch", 4, "batch_micro_kernel"): 313169661,      # profiles/hbm_traffic_resnet18_batch.md (levels switching)
}

# Counted traffic of all kernels of one step (sum of the per-kernel averages in the same summaries;
# kernels that run once per window or on demand left out).  Key: (workload, W).
MEASURED_STEP_TRAFFIC_BYTES = {
    ("resnet18_topk", 4): 657244796 + 267390242 + 28096254 + 9426446 + 2466338 + 2097376,
    ("resnet18_powersgd", 4): 635250034 + 191304669 + 12184522 + 3387700 + 47511470,
    ("vgg19_powersgd", 1): 416681243 + 88425680 + 6209777 + 1803930 + 86544871,
    ("lstm_topk", 16): 10615536735 + 4250833287 + 453200928 + 143393238 + 30725046 + 11360930 + 4826538,
    ("resnet18_topk_k99", 4): 637193697 + 436029832 + 19702033 + 5225139 + 2109252 + 2458557,
}

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


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "the path would shard by worker (one data-parallel worker per GPU)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2010_16248_amd import binding as B
    from paper_2010_16248_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load_library()                       # fails loudly if the HIP library is missing
    w = wl.workload(args.workload)
    W = args.workers if args.workers > 0 else w.n_workers
    layers = w.layers
    N = w.n_params
    rmax = max(w.level_crit, w.level_noncrit)
    q0 = wl.q_init(w, rmax, w.seed) if w.method == B.ACC_POWERSGD else None
    is_batch = w.method == B.ACC_BATCH
    gpu = B.Accordion(w.method, layers, W, w.level_crit, w.level_noncrit, w.k_den, w.eta, 1, q0,
                      batch_multiplier=w.batch_multiplier)

    # gradient pool, resident in HBM: [scale][batch][worker]
    dev = torch.device("cuda:0")
    base = [[torch.from_numpy(wl.gradient(w, k, s)).to(dev) for k in range(W)] for s in range(args.pool)]
    out = torch.empty(N, dtype=torch.float32, device=dev)
    weights = velocity = None
    if args.fused_update:
        weights = torch.full((N,), 0.01, dtype=torch.float32, device=dev)
        velocity = torch.zeros(N, dtype=torch.float32, device=dev)
    if args.fixed_level in (0, 1):
        st = gpu.unpack_state(gpu.get_state())
        blob = gpu.pack_state(st["e"], st["A"], st["Q"], st["norm_old"], st["has_old"],
                              np.full(gpu.n_layers, args.fixed_level, np.int32), 0)
        gpu.set_state(blob)

    # plain copy of known size: the copy bandwidth this machine reaches, and the kernel that calibrates
    # FETCH_SIZE / WRITE_SIZE in a rocprofv3 --pmc run of this file
    copy_probe = None
    if args.probe_mib > 0:
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

    state = {"step": 0}
    graphs = None
    if args.hip_graph:
        args.kernel_events = "none"
        if is_batch and args.pool % 2:
            print("bench.py: --hip-graph in batch-size mode needs an even --pool", file=sys.stderr)
            sys.exit(2)

    def one_step():
        s = state["step"]
        if graphs is not None:
            graphs[s % args.pool].replay()
        elif args.fused_update:
            gpu.step_all_update(base[s % args.pool], weights, velocity, LR_CURR, 0.9, 0.0)
        else:
            gpu.step_all(base[s % args.pool], out)
        if args.fixed_level < 0 and (s + 1) % args.window == 0:
            # every second window ends with an LR decay (not in batch-size mode, where the large
            # batch, once reached, is kept: the timed region is the steady state)
            decay = ((s + 1) // args.window) % 2 == 1 and not is_batch
            gpu.detect_regime(LR_CURR, LR_CURR * 0.1 if decay else LR_CURR)
        state["step"] = s + 1

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    if args.hip_graph:
        # steady state reached: capture one step per pool batch on a side stream
        side = torch.cuda.Stream()
        gpu.set_stream(side.cuda_stream)
        captured = []
        for b in range(args.pool):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                if args.fused_update:
                    gpu.step_all_update(base[b], weights, velocity, LR_CURR, 0.9, 0.0)
                else:
                    gpu.step_all(base[b], out)
            captured.append(g)
        graphs = captured
        torch.cuda.synchronize()
        gpu.set_stream(torch.cuda.current_stream().cuda_stream)   # replays and eager calls share a stream
    state["step"] = 0                      # timed region starts at a window boundary
    use_events = args.kernel_events != "none"
    if use_events:
        gpu.set_profiling({"all": 1, "dominant": 2, "sampled": 3}[args.kernel_events])
    torch.cuda.synchronize()
    bs0 = gpu.batch_status() if is_batch else None
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    gpu.flush()                            # PowerSGD: the last step's residual is written out
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = gpu.get_profile() if use_events else {}
    if use_events:
        gpu.set_profiling(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = 4.0 * N * W / (ms_per_step * 1e-3) / 1e9

    levels = gpu.get_levels()
    words_last, words_cum = gpu.payload_words()

    dom = dominant_kernel(w.method)
    roofline = None
    kernels = {}
    if prof:
        tot = sum(ms for ms, _ in prof.values())
        for name, (ms, n) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            kernels[name] = {"avg_us": round(ms * 1e3 / n, 2), "launches": n, "share": round(ms / tot, 3)}
        if is_batch and args.fused_update:
            dom = "batch_micro_update_kernel"
        ms, n = prof[dom]
        avg_s = ms * 1e-3 / n
        if is_batch:
            bs1 = gpu.batch_status()
            steps_t, exch_t = bs1["micro_steps"] - bs0["micro_steps"], bs1["exchanges"] - bs0["exchanges"]
            alg_bytes = algorithmic_bytes_batch(N, W, steps_t, exch_t) // max(1, steps_t)
            if args.fused_update:
                alg_bytes += 12 * N * exch_t // max(1, steps_t)     # w, v read and written, no D store
        else:
            alg_bytes = algorithmic_bytes_dominant(N, W)
        ach = alg_bytes / avg_s / 1e9
        traffic = MEASURED_TRAFFIC_BYTES.get((args.workload, W, dom))
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "avg_kernel_us": round(avg_s * 1e6, 2), "launches_timed": n,
                    "algorithmic_bytes_per_launch": alg_bytes}

    # the whole step: bytes the method must move (one read / write of each operand per pass, the
    # payload at the level of the last step) and the traffic counted by rocprofv3 for all kernels
    step_bw = None
    if not is_batch:
        alg = algorithmic_bytes_step(w, layers, W, [words_last // 2])
        cnt = MEASURED_STEP_TRAFFIC_BYTES.get((args.workload, W))
        if args.fused_update:                # weights and velocity read and written instead of D written
            alg += 12 * N
            cnt = None                       # counted for the storing sink only
        step_bw = {"algorithmic_bytes": alg, "algorithmic_GB/s": round(alg / (ms_per_step * 1e-3) / 1e9, 1),
                   "counted_bytes": cnt,
                   "counted_GB/s": round(cnt / (ms_per_step * 1e-3) / 1e9, 1) if cnt else None,
                   "counted_frac_of_peak": round(cnt / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if cnt else None}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, W, 400, args.window)

    line = {
        "metric": "gradient GB/s per compress step (EF+compress+norm)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_params": N, "n_workers": W, "n_layers": len(layers),
                   "method": {B.ACC_TOPK: "topk", B.ACC_POWERSGD: "powersgd", B.ACC_BATCH: "batch"}[w.method],
                   "batch_multiplier": w.batch_multiplier,
                   "level_crit": w.level_crit, "level_noncrit": w.level_noncrit,
                   "window_steps": args.window, "pool_batches": args.pool,
                   "levels_switch": args.fixed_level < 0, "hip_graph": bool(args.hip_graph),
                   "sink": "nesterov update of weights and velocity" if args.fused_update else "averaged gradient stored", "kernel_events_in_timed_region": args.kernel_events},
        "roofline": roofline,
        "step_bandwidth": step_bw,
        "cpu_baseline": cpu,
        "copy_probe": copy_probe,
        "kernels": kernels,
        "payload_words_last_step": words_last,
        "critical_layers_at_end": int(levels.sum()),
    }
    gpu.destroy()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
