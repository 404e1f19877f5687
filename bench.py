#!/usr/bin/env python3
"""Benchmark of the CheckFree recovery hot path on one MI355X.

A *step* is one pass of the whole path over one synthetic workload: squared
gradient norms of the neighbouring stages in one launch, then the fused
norm-to-weight scaling + weighted-average blend into the lost stage (workloads
1, 2, 3, 5), or the CheckFree+ copy (workload 4).  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-cpu-baseline] [--no-ceilings]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure

# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE counters, each scaled by what the same
# counter reads for the copy kernel of known size (profiles/cf_kernels_hbm_traffic_pmc.md).  Valid only
# for the kernel sources they were taken on: reported as null once those have changed.
TRAFFIC_KERNEL_SHA256 = "3b9084d45d82213f7b2b39c1f8a5d0146f060b5f1f005929d2564a57beded7d2"
TRAFFIC_BYTES_PER_LAUNCH = {(3, "cf_blend_kernel"): 2464870000}


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for name in ("cf_kernels.hip", "cf_kernels.h"):
        with open(os.path.join(ROOT, "paper_2506_15461_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = the 1.5B-shape stage the metric is quoted on)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-ceilings", action="store_true",
                   help="skip the read-only / copy ceiling measurements (keeps a profile to the timed kernels)")
    p.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline")
    p.add_argument("--shape", type=str, default=None, help="override the stage shape: d,ffn,layers (exploration only)")
    p.add_argument("--sets", type=int, default=0,
                   help="independent buffer sets rotated step by step so that no step finds its inputs in the "
                        "256 MB Infinity Cache (0 = enough sets to cover 1.5 GB)")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this library runs on exactly one GPU (asked for {args.gpus}); "
              "the path has no multi-GPU leg.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2506_15461_amd as cf
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cf.load_library()                      # fails loudly if the HIP library is not built
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    spec = workloads.SPECS[args.config]
    shape = None
    if args.shape:
        d, ffn, layers = (int(x) for x in args.shape.split(","))
        shape = workloads.StageShape(d, ffn, layers)
    ctx = cf.Context(0)
    stream = torch.cuda.current_stream()

    def build_set(wl):
        """Stage handles and the step closure for one set of buffers."""
        if args.config == 4:
            src_t = wl.weights[0] + wl.extra
            dst_t = [torch.full_like(t, float("nan")) for t in src_t]
            src, dst = cf.Stage(ctx, src_t), cf.Stage(ctx, dst_t)

            def step(ev=None):
                if ev:
                    ev[0].record(stream)
                cf.cf_copy_stage(ctx, src, dst, stream)
                if ev:
                    ev[1].record(stream)
            return step, {"copy": 2 * src.nbytes}, (src, dst, dst_t)
        if args.config == 5:
            lost = wl.lost
            grad_stages = [cf.Stage(ctx, g) for g in wl.grads]
            ip, inx = lost - 1, lost + 1
        else:
            lost = 1
            grad_stages = [cf.Stage(ctx, wl.grads[0]), cf.Stage(ctx, wl.grads[2])]
            ip, inx = 0, 1
        prev, nxt, out = (cf.Stage(ctx, wl.weights[i]) for i in (lost - 1, lost + 1, lost))
        omega = torch.zeros(len(grad_stages), dtype=torch.float64, device=dev)
        w_prev, w_next = omega[ip:ip + 1], omega[inx:inx + 1]

        def step(ev=None):
            if ev:
                ev[0].record(stream)
            cf.cf_stage_grad_sqnorm(ctx, grad_stages, omega, stream)
            if ev:
                ev[1].record(stream)
            cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, w_prev, w_next, out, stream)
            if ev:
                ev[2].record(stream)
        return step, {"sqnorm": sum(g.nbytes for g in grad_stages), "blend": 3 * out.nbytes}, (grad_stages, prev, nxt, out, omega)

    wl = workloads.make_workload(args.config, device=dev, shape=shape, with_grads=args.config != 4)
    spec = wl.spec
    numel = spec.shape.numel()
    step0, kernel_bytes, keep0 = build_set(wl)
    step_bytes = sum(kernel_bytes.values())
    kernels = list(kernel_bytes)
    dominant = "copy" if args.config == 4 else "blend"
    # Rotate over enough independent buffer sets that a step never finds its
    # inputs in the 256 MB Infinity Cache left there by the step before.
    n_sets = args.sets if args.sets > 0 else max(1, -(-int(1.5e9) // step_bytes))
    steps_fn, keep = [step0], [keep0, wl]
    for i in range(1, n_sets):
        wl_i = workloads.make_workload(args.config, device=dev, shape=shape, seed=spec.seed + 1000 * i,
                                       with_grads=args.config != 4)
        st, _, kp = build_set(wl_i)
        steps_fn.append(st)
        keep += [kp, wl_i]

    def step(k, ev=None):
        steps_fn[k % n_sets](ev)

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    # HIP events on the launch stream, inside the timed region, around each kernel of every
    # `sample_every`-th step (about 40 samples): an event record costs ~3.5 us of dispatch time on
    # this stack, so bracketing every kernel of every step would inflate the step by 1.7 %.
    sample_every = max(1, args.steps // 40)
    sampled = [k for k in range(args.steps) if k % sample_every == 0]
    events = {k: [torch.cuda.Event(enable_timing=True) for _ in range(len(kernels) + 1)] for k in sampled}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k, events.get(k))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flags = ctx.read_flags()

    kernel_ms = {}
    for j, name in enumerate(kernels):
        d = np.array([events[k][j].elapsed_time(events[k][j + 1]) for k in sampled])
        kernel_ms[name] = {"avg": float(d.mean()), "median": float(np.median(d)), "min": float(d.min())}
    d = np.array([events[k][0].elapsed_time(events[k][-1]) for k in sampled])
    sampled_step = {"median": round(float(np.median(d)), 5), "min": round(float(d.min()), 5), "n": len(sampled)}
    gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    dom_ms = kernel_ms[dominant]["avg"]
    achieved = kernel_bytes[dominant] / (dom_ms * 1e-3) / 1e9

    dominant_kernel = {"blend": "cf_blend_kernel", "copy": "cf_copy_kernel"}[dominant]
    traffic = None
    if not args.shape and kernel_sources_sha256() == TRAFFIC_KERNEL_SHA256:
        traffic = TRAFFIC_BYTES_PER_LAUNCH.get((args.config, dominant_kernel))

    result = {
        "metric": "stage_recovery_achieved_hbm_bandwidth",
        "stage_recovery_ms": round(ms_per_step, 5),
        "sampled_step_ms": sampled_step,
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {
            "workload": f"config {args.config}: {spec.name}",
            "stage": {"d": spec.shape.d, "ffn": spec.shape.ffn, "layers": spec.shape.layers,
                      "tensors": len(spec.shape.tensor_shapes()), "numel": numel},
            "weight_dtype": spec.param_dtype, "grad_dtype": "f32",
            "step": "+".join(kernels),
            "algorithmic_bytes_per_step": int(step_bytes),
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "buffer_sets_rotated": n_sets,
            "steps_with_kernel_events": len(sampled),
            "device_flags": flags,
        },
        "kernels": {name: {"ms_avg": round(v["avg"], 5), "ms_median": round(v["median"], 5),
                           "ms_min": round(v["min"], 5),
                           "GBps_avg": round(kernel_bytes[name] / (v["avg"] * 1e-3) / 1e9, 1)}
                    for name, v in kernel_ms.items()},
        "roofline": {
            "kernel": dominant_kernel,
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by the copy kernel's)",
            "algorithmic_bytes_per_launch": int(kernel_bytes[dominant]),
        },
    }

    if not args.no_ceilings:
        result["ceilings"] = measure_ceilings(args, wl, ctx, cf, torch, stream)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, wl, step_bytes, torch, workloads)
    print(json.dumps(result), flush=True)
    return 0


def measure_ceilings(args, wl, ctx, cf, torch, stream, reps=20):
    """What this machine sustains on one stage's worth of data (outside the timed region): a read-only
    stream (the norm's first and second pass), this library's copy, and PyTorch's device-to-device
    copy of the same tensors (the runtime's own copy kernel) as an outside reference."""
    src_t = wl.weights[0] + wl.extra if args.config == 4 else wl.weights[wl.lost - 1]
    dst_t = [torch.empty_like(t) for t in src_t]
    src, dst = cf.Stage(ctx, src_t), cf.Stage(ctx, dst_t)
    nbytes = src.nbytes
    omega = torch.zeros(1, dtype=torch.float64, device=src_t[0].device)
    readable = all(t.dtype in (torch.float32, torch.bfloat16) for t in src_t)

    def timed(fn):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {"bytes_per_stream": int(nbytes)}
    if readable:
        ms = timed(lambda: cf.cf_stage_grad_sqnorm(ctx, [src], omega, stream))
        out["read_only_GBps"] = round(nbytes / ms / 1e6, 1)
    ms = timed(lambda: cf.cf_copy_stage(ctx, src, dst, stream))
    out["copy_GBps"] = round(2 * nbytes / ms / 1e6, 1)
    ms = timed(lambda: torch._foreach_copy_(dst_t, src_t))
    out["torch_foreach_copy_GBps"] = round(2 * nbytes / ms / 1e6, 1)
    flat_s = torch.empty(nbytes // 4, dtype=torch.float32, device=src_t[0].device).normal_()
    flat_d = torch.empty_like(flat_s)
    ms = timed(lambda: flat_d.copy_(flat_s))
    out["torch_flat_copy_GBps"] = round(2 * flat_s.numel() * 4 / ms / 1e6, 1)
    return out


def cpu_baseline(args, wl, step_bytes, torch, workloads):
    """The oracle, as it stands, on this host's cores, over the same workload
    (or a bounded part of it), repeated until about --cpu-seconds have passed."""
    import oracle
    threads = max(1, min(oracle.max_threads(), os.cpu_count() or 1))
    if args.config == 4:
        src = [workloads.to_numpy(t) for t in wl.weights[0] + wl.extra]
        nbytes = 2 * sum(a.nbytes for a in src)
        sample = "whole workload (39 tensors)"

        def cpu_step():
            oracle.copy_stage(src, threads)
    else:
        lost = wl.lost
        if args.config == 5:
            gidx = list(range(len(wl.grads)))
        else:
            gidx = [0, 2]
        grads = [workloads.stage_to_numpy(wl.grads[i]) for i in gidx]
        prev = workloads.stage_to_numpy(wl.weights[lost - 1])
        nxt = workloads.stage_to_numpy(wl.weights[lost + 1])
        nbytes = step_bytes
        sample = "whole workload, same tensors as the GPU step"

        def cpu_step():
            om = [oracle.stage_grad_sqnorm(g, threads) for g in grads]
            ip, inx = (lost - 1, lost + 1) if args.config == 5 else (0, 1)
            oracle.recover_stage_weighted_avg(prev, nxt, om[ip], om[inx], threads)
    t0 = time.perf_counter()
    reps = 0
    while True:
        cpu_step()
        reps += 1
        el = time.perf_counter() - t0
        if el * threads >= args.cpu_seconds or reps >= 50:
            break
    sec = el / reps
    out = {"value": round(nbytes / sec / 1e9, 2), "unit": "GB/s", "cores": threads, "kind": "oracle",
           "ms_per_step": round(sec * 1e3, 2),
           "sample": f"{sample}; {reps} repetition(s), {el:.1f} s wall on {threads} thread(s)"}
    if threads > 1:
        # the same step once on a single thread, for scale
        threads = 1
        t0 = time.perf_counter()
        cpu_step()
        sec1 = time.perf_counter() - t0
        out["single_thread"] = {"value": round(nbytes / sec1 / 1e9, 2), "unit": "GB/s", "ms_per_step": round(sec1 * 1e3, 1)}
    out["host"] = {"cpu_model": cpu_model(), "logical_cpus": os.cpu_count()}
    return out


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


if __name__ == "__main__":
    sys.exit(main())
