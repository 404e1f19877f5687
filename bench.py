#!/usr/bin/env python3
"""Benchmark of the CheckFree recovery hot path on one MI355X.

A *step* is one pass of the whole path over one synthetic workload: squared
gradient norms of the neighbouring stages in one launch, then the fused
norm-to-weight scaling + weighted-average blend into the lost stage (workloads
1, 2, 3, 5), or the CheckFree+ copy (workload 4).  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

The headline fields are those of --config (default 3, the 1.5B-shape stage the
metric is quoted on).  With the default configuration the same line also carries
    per_config    the other four workloads, shorter runs of the same step
    graph_replay  the same step replayed from a captured HIP graph
    setup         cost of creating the five stage handles of a recovery, in
                  library-allocated and in caller-provided memory, and a recovery
                  timed from before the handles exist
    optimizer_step  one stage's Adam step that also yields omega (no separate read of the gradients)
    replica_refresh (with --config 4) embedding + de-embedding refresh, whole and in slices
    ceilings      what two trivial kernels (flat buffer, no table) sustain on this GPU
    cpu_baseline  the CPU oracle on the host's cores

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
                    [--no-cpu-baseline] [--no-ceilings] [--no-per-config] [--no-setup] [--no-graph]
    python bench.py --size-sweep      (another line: the three kernels from 4 MiB to 2 GiB per stream)
"""
import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor figure

# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE counters, each
# scaled by what the same counter reads for a plain copy kernel of known size; STORED from the
# profile named below, not measured in this run, and valid only for the kernel sources it was taken
# on: reported as null once those have changed.
TRAFFIC_PROFILE = "profiles/cf_kernels_hbm_traffic_pmc.md"
TRAFFIC_KERNEL_SHA256 = "b001382d9ee5de9dedbba6b64b36fbf2daa43f39ef5ecadf83ee183af2fd8eec"
TRAFFIC_BYTES_PER_LAUNCH = {(3, "cf_blend_kernel"): 2471127000}


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for name in ("cf_kernels.hip", "cf_kernels.h", "cf_device.h"):
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
    p.add_argument("--no-per-config", action="store_true", help="skip the short runs of the other four workloads")
    p.add_argument("--no-setup", action="store_true", help="skip the handle-creation timings")
    p.add_argument("--no-graph", action="store_true", help="skip the graph-replayed step")
    p.add_argument("--only-step", action="store_true",
                   help="the timed steps and nothing else (for profiling): implies all --no-* switches")
    p.add_argument("--size-sweep", action="store_true",
                   help="instead of the benchmark: bandwidth of the norm, the blend (fp32, bf16) and the copy for "
                        "single-tensor stages of 4 MiB .. 2 GiB, cold rotating buffer sets; prints one JSON line")
    p.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline")
    p.add_argument("--shape", type=str, default=None, help="override the stage shape: d,ffn,layers (exploration only)")
    p.add_argument("--sets", type=int, default=0,
                   help="independent buffer sets rotated step by step so that no step finds its inputs in the "
                        "256 MB Infinity Cache (0 = enough sets to cover 1.5 GB)")
    p.add_argument("--sqnorm-blocks-per-cu", type=int, default=0, help="tuning knob of the norm's first pass (0 = default)")
    p.add_argument("--chunk-bytes", type=int, default=0, help="tuning knob: bytes per work chunk (0 = default)")
    args = p.parse_args()
    if args.only_step:
        args.no_cpu_baseline = args.no_ceilings = args.no_per_config = args.no_setup = args.no_graph = True
    return args


class Runner:
    """One workload resident on the GPU: its buffer sets, stage handles and the step."""

    def __init__(self, config, args, ctx, cf, torch, workloads, shape=None):
        self.config, self.ctx, self.cf, self.torch = config, ctx, cf, torch
        dev = ctx.device
        self.stream = torch.cuda.current_stream()
        self.wl = workloads.make_workload(config, device=dev, shape=shape, with_grads=config != 4)
        self.spec = self.wl.spec
        step0, self.kernel_bytes, keep0 = self._build_set(self.wl)
        self.step_bytes = sum(self.kernel_bytes.values())
        self.kernels = list(self.kernel_bytes)
        self.dominant = "copy" if config == 4 else "blend"
        # Rotate over enough independent buffer sets that a step never finds its inputs in the
        # 256 MB Infinity Cache left there by the step before.
        self.n_sets = args.sets if args.sets > 0 else max(1, -(-int(1.5e9) // self.step_bytes))
        self.steps_fn, self.keep = [step0], [keep0]
        for i in range(1, self.n_sets):
            wl_i = workloads.make_workload(config, device=dev, shape=shape, seed=self.spec.seed + 1000 * i,
                                           with_grads=config != 4)
            st, _, kp = self._build_set(wl_i)
            self.steps_fn.append(st)
            self.keep += [kp, wl_i]
        torch.cuda.synchronize()

    def _build_set(self, wl):
        cf, ctx, torch, stream = self.cf, self.ctx, self.torch, self.stream
        if self.config == 4:
            src_t = wl.weights[0] + wl.extra
            dst_t = [torch.full_like(t, float("nan")) for t in src_t]
            src, dst = cf.Stage(ctx, src_t), cf.Stage(ctx, dst_t)

            def step(ev=None, stream=stream):
                if ev:
                    ev[0].record(stream)
                cf.cf_copy_stage(ctx, src, dst, stream)
                if ev:
                    ev[1].record(stream)
            return step, {"copy": 2 * src.nbytes}, (src, dst, dst_t)
        if self.config == 5:
            lost = wl.lost
            grad_stages = [cf.Stage(ctx, g) for g in wl.grads]
            ip, inx = lost - 1, lost + 1
        else:
            lost = 1
            grad_stages = [cf.Stage(ctx, wl.grads[0]), cf.Stage(ctx, wl.grads[2])]
            ip, inx = 0, 1
        prev, nxt, out = (cf.Stage(ctx, wl.weights[i]) for i in (lost - 1, lost + 1, lost))
        omega = torch.zeros(len(grad_stages), dtype=torch.float64, device=ctx.device)
        w_prev, w_next = omega[ip:ip + 1], omega[inx:inx + 1]

        def step(ev=None, stream=stream):
            if ev:
                ev[0].record(stream)
            cf.cf_stage_grad_sqnorm(ctx, grad_stages, omega, stream)
            if ev:
                ev[1].record(stream)
            cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, w_prev, w_next, out, stream)
            if ev:
                ev[2].record(stream)
        return step, {"sqnorm": sum(g.nbytes for g in grad_stages), "blend": 3 * out.nbytes}, \
            (grad_stages, prev, nxt, out, omega)

    def step(self, k, ev=None):
        self.steps_fn[k % self.n_sets](ev)

    def time_steps(self, steps, warmup):
        """Wall time of `steps` back-to-back steps; HIP events on the launch stream, inside the timed
        region, around each kernel of every `sample_every`-th step (every fifth step at least, about 40
        samples in a long run): an event record costs ~3.5 us of dispatch time on this stack, so
        bracketing every kernel of every step would inflate a short step noticeably."""
        import numpy as np
        torch = self.torch
        for k in range(warmup):
            self.step(k)
        torch.cuda.synchronize()
        sample_every = max(5, steps // 40) if steps >= 10 else 1
        sampled = [k for k in range(steps) if k % sample_every == 0]
        events = {k: [torch.cuda.Event(enable_timing=True) for _ in range(len(self.kernels) + 1)] for k in sampled}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(k, events.get(k))
        t_enqueued = time.perf_counter()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        self.host_enqueue_ms_per_step = (t_enqueued - t0) * 1e3 / steps
        kernel_ms = {}
        for j, name in enumerate(self.kernels):
            d = np.array([events[k][j].elapsed_time(events[k][j + 1]) for k in sampled])
            kernel_ms[name] = {"avg": float(d.mean()), "median": float(np.median(d)), "min": float(d.min())}
        d = np.array([events[k][0].elapsed_time(events[k][-1]) for k in sampled])
        sampled_step = {"median": round(float(np.median(d)), 5), "min": round(float(d.min()), 5), "n": len(sampled)}
        return ms_per_step, kernel_ms, sampled_step

    def time_graph(self, steps):
        """The same steps captured once in a HIP graph (one step per buffer set) and replayed: what is
        left of a step when the host's launch work is out of the way."""
        torch = self.torch
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for fn in self.steps_fn:
                fn(None, side)
            side.synchronize()
            graph.capture_begin()
            for fn in self.steps_fn:
                fn(None, side)
            graph.capture_end()
        torch.cuda.synchronize()
        replays = max(2, -(-steps // self.n_sets))
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / (replays * self.n_sets)
        return {"ms_per_step": round(ms, 5), "GBps": round(self.step_bytes / ms / 1e6, 1),
                "frac_of_hbm_peak": round(self.step_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                "steps": replays * self.n_sets, "steps_per_graph": self.n_sets}

    def kernel_table(self, kernel_ms):
        return {name: {"ms_avg": round(v["avg"], 5), "ms_median": round(v["median"], 5), "ms_min": round(v["min"], 5),
                       "GBps_avg": round(self.kernel_bytes[name] / (v["avg"] * 1e-3) / 1e9, 1)}
                for name, v in kernel_ms.items()}

    def close(self):
        self.steps_fn, self.keep, self.wl = [], [], None
        gc.collect()
        self.torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this library runs on exactly one GPU (asked for {args.gpus}); "
              "the path has no multi-GPU leg.", file=sys.stderr)
        return 2

    import torch

    import paper_2506_15461_amd as cf
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cf.load_library()                      # fails loudly if the HIP library is not built
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    shape = None
    if args.shape:
        d, ffn, layers = (int(x) for x in args.shape.split(","))
        shape = workloads.StageShape(d, ffn, layers)
    tuning = {}
    if args.sqnorm_blocks_per_cu:
        tuning["sqnorm_blocks_per_cu"] = args.sqnorm_blocks_per_cu
    if args.chunk_bytes:
        tuning["chunk_bytes"] = args.chunk_bytes
    ctx = cf.Context(0, **tuning)
    if args.size_sweep:
        print(json.dumps(size_sweep(ctx, cf, torch)))
        return 0

    run = Runner(args.config, args, ctx, cf, torch, workloads, shape)
    spec = run.spec
    # The ceilings are measured first: on different buffers, outside the timed region, and they leave the
    # GPU at its working clocks when the W warm-up steps begin (after the host-bound set-up the first
    # 20 or so steps otherwise run up to 5 % slow, which a short run would average in).
    ceilings = None if args.no_ceilings else measure_ceilings(args, run, ctx, cf, torch)
    ms_per_step, kernel_ms, sampled_step = run.time_steps(args.steps, args.warmup)
    flags = ctx.read_flags()
    gbps = run.step_bytes / (ms_per_step * 1e-3) / 1e9
    dominant = run.dominant
    achieved = run.kernel_bytes[dominant] / (kernel_ms[dominant]["avg"] * 1e-3) / 1e9
    dominant_kernel = {"blend": "cf_blend_kernel", "copy": "cf_copy_kernel"}[dominant]
    traffic = None
    if not args.shape and not tuning and kernel_sources_sha256() == TRAFFIC_KERNEL_SHA256:
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
                      "tensors": len(spec.shape.tensor_shapes()), "numel": spec.shape.numel()},
            "weight_dtype": spec.param_dtype, "grad_dtype": "f32",
            "step": "+".join(run.kernels),
            "algorithmic_bytes_per_step": int(run.step_bytes),
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "buffer_sets_rotated": run.n_sets,
            "steps_with_kernel_events": sampled_step["n"],
            "device_flags": flags,
            "host_enqueue_ms_per_step": round(run.host_enqueue_ms_per_step, 5),
            "tuning": tuning or "default",
        },
        "kernels": run.kernel_table(kernel_ms),
        "roofline": {
            "kernel": dominant_kernel,
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy kernel's)",
            "traffic_source": f"stored from {TRAFFIC_PROFILE}, not measured in this run; null when the kernel sources "
                              "have changed since",
            "algorithmic_bytes_per_launch": int(run.kernel_bytes[dominant]),
        },
    }

    if not args.no_graph:
        result["graph_replay"] = run.time_graph(args.steps)
    if not args.no_setup and args.config in (1, 2, 3):
        result["setup"] = measure_setup(run, ctx, cf, torch)
    if args.config == 4 and not args.no_setup:
        result["replica_refresh"] = measure_replica_refresh(run, ctx, cf, torch)
    if args.config != 4 and not args.no_setup:
        result["optimizer_step"] = measure_optimizer_step(run, ctx, cf, torch)
    if ceilings is not None:
        result["ceilings"] = ceilings
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, run.wl, run.step_bytes, torch, workloads)

    if not args.no_per_config and args.config == 3 and not args.shape:
        run.close()
        per = {}
        # (steps, warm-up steps): about 30 ms of warm-up each, so that the clocks have settled after the
        # host-bound construction of the workload, and at least 50 ms timed
        plan = {1: (1000, 600), 2: (500, 300), 4: (150, 80), 5: (60, 30)}
        for c in (1, 2, 4, 5):
            steps, warm = plan[c]
            r = Runner(c, args, ctx, cf, torch, workloads)
            ms, kms, _ = r.time_steps(steps, warm)
            entry = {"workload": r.spec.name, "ms_per_step": round(ms, 5), "GBps": round(r.step_bytes / ms / 1e6, 1),
                     "frac_of_hbm_peak": round(r.step_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_step": int(r.step_bytes), "steps": steps, "buffer_sets_rotated": r.n_sets,
                     "host_enqueue_ms_per_step": round(r.host_enqueue_ms_per_step, 5),
                     "kernels": {k: {"ms_avg": v["ms_avg"], "GBps_avg": v["GBps_avg"]}
                                 for k, v in r.kernel_table(kms).items()}}
            if not args.no_graph:
                g = r.time_graph(steps)
                entry["graph_replay"] = {"ms_per_step": g["ms_per_step"], "frac_of_hbm_peak": g["frac_of_hbm_peak"]}
            if c == 4 and not args.no_setup:
                entry["replica_refresh"] = measure_replica_refresh(r, ctx, cf, torch)
            per[str(c)] = entry
            r.close()
        result["per_config"] = per
        result["per_config_device_flags"] = ctx.read_flags()
    print(json.dumps(result), flush=True)
    return 0


def measure_setup(run, ctx, cf, torch, reps=15):
    """Creating the five stage handles a recovery needs (gradients of both neighbours, weights of both
    neighbours, the lost stage) -- what a joining node does right after it has received its neighbours'
    stages -- through the C ABI with the descriptors already marshalled:
      library_allocated   cf_stage_create x 5: hipMalloc + table kernel + wait, each
      caller_memory       cf_stage_create_in x 5 into preallocated torch memory on the stream: host time
                          to enqueue, and time until the tables are complete on the device
    and one recovery (handles + norms + blend) timed from before the handles exist until the lost stage
    is written, both ways."""
    import numpy as np
    lib = cf.load_library()
    wl = run.wl
    lists = [wl.grads[0], wl.grads[2], wl.weights[0], wl.weights[2], wl.weights[1]]
    descs = [cf.tensor_descriptors(l) for l in lists]
    counts = [len(l) for l in lists]
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    nbytes = [int(lib.cf_stage_table_bytes(ctx._h, d, n)) for d, n in zip(descs, counts)]
    tables = [torch.empty(b, dtype=torch.uint8, device=ctx.device) for b in nbytes]
    omega = torch.zeros(2, dtype=torch.float64, device=ctx.device)
    om = [ctypes.c_void_p(omega.data_ptr()), ctypes.c_void_p(omega.data_ptr() + 8)]

    def create_owned():
        hs = []
        for d, n in zip(descs, counts):
            h = ctypes.c_void_p()
            assert lib.cf_stage_create(ctx._h, d, n, ctypes.byref(h)) == 0
            hs.append(h)
        return hs

    def create_in():
        hs = []
        for d, n, t, b in zip(descs, counts, tables, nbytes):
            h = ctypes.c_void_p()
            assert lib.cf_stage_create_in(ctx._h, d, n, ctypes.c_void_p(t.data_ptr()), b, sp, ctypes.byref(h)) == 0
            hs.append(h)
        return hs

    def recover(hs):
        grads = (ctypes.c_void_p * 2)(hs[0], hs[1])
        assert lib.cf_stage_grad_sqnorm(ctx._h, grads, 2, om[0], sp) == 0
        assert lib.cf_recover_stage_weighted_avg(ctx._h, hs[2], hs[3], om[0], om[1], hs[4], sp) == 0

    def destroy(hs):
        for h in hs:
            lib.cf_stage_destroy(h)

    t_owned, t_enq, t_ready, r_owned, r_in = [], [], [], [], []
    for rep in range(reps + 2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hs = create_owned()
        t1 = time.perf_counter()
        destroy(hs)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        hs = create_in()
        t3 = time.perf_counter()
        stream.synchronize()
        t4 = time.perf_counter()
        destroy(hs)
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        hs = create_owned()
        recover(hs)
        stream.synchronize()
        t6 = time.perf_counter()
        destroy(hs)
        torch.cuda.synchronize()
        t7 = time.perf_counter()
        hs = create_in()
        recover(hs)
        stream.synchronize()
        t8 = time.perf_counter()
        destroy(hs)
        if rep >= 2:
            t_owned.append(t1 - t0), t_enq.append(t3 - t2), t_ready.append(t4 - t2)
            r_owned.append(t6 - t5), r_in.append(t8 - t7)

    def med(x):
        return round(float(np.median(x)) * 1e3, 4)
    return {
        "what": "5 stage handles of one recovery (2 gradient stages, 2 neighbour stages, the lost stage), "
                f"{counts[0]} tensors each; C ABI calls with descriptors already marshalled; medians of {reps}",
        "table_bytes_per_stage": nbytes[0],
        "library_allocated_ms": med(t_owned),
        "caller_memory_enqueue_ms": med(t_enq),
        "caller_memory_ready_ms": med(t_ready),
        "recovery_incl_setup_library_allocated_ms": med(r_owned),
        "recovery_incl_setup_caller_memory_ms": med(r_in),
    }


def measure_optimizer_step(run, ctx, cf, torch, reps=20):
    """Steady state: every stage keeps omega of its last gradient.  One stage's Adam step with omega as a
    by-product (cf_adam_step_with_sqnorm: 4 reads + 3 writes of 4 bytes per element, nothing else), beside
    the dedicated norm of the same gradients (what keeping omega current costs without the fused pass)."""
    wl = run.wl
    stream = torch.cuda.current_stream()
    w = [t.clone() for t in wl.weights[wl.lost - 1]]
    if w[0].dtype != torch.float32:
        w = [t.float() for t in w]
    g = wl.grads[wl.lost - 1]
    m = [torch.zeros_like(t) for t in w]
    v = [torch.zeros_like(t) for t in w]
    sw, sm, sv, sg = (cf.Stage(ctx, x) for x in (w, m, v, g))
    scratch = torch.empty(cf.adam_scratch_bytes(sg), dtype=torch.uint8, device=ctx.device)
    omega = torch.zeros(1, dtype=torch.float64, device=ctx.device)
    omega2 = torch.zeros(1, dtype=torch.float64, device=ctx.device)
    step = [0]

    def fused():
        step[0] += 1
        cf.cf_adam_step_with_sqnorm(ctx, sw, sm, sv, sg, 3e-4, 0.9, 0.999, 1e-8, step[0], scratch, omega, stream)

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

    ms = timed(fused)
    ms_norm = timed(lambda: cf.cf_stage_grad_sqnorm(ctx, [sg], omega2, stream))
    nbytes = 28 * sg.numel
    torch.cuda.synchronize()
    rel = abs(omega.item() - omega2.item()) / max(omega2.item(), 1e-300)
    return {"what": "Adam step of one stage with omega as a by-product (cf_adam_step_with_sqnorm); fp32 weights, "
                    "moments and gradients",
            "elements": sg.numel, "algorithmic_bytes": nbytes, "ms": round(ms, 5), "GBps": round(nbytes / ms / 1e6, 1),
            "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
            "dedicated_norm_of_the_same_gradients_ms": round(ms_norm, 5),
            "omega_relative_difference_to_dedicated_norm": rel}


def measure_replica_refresh(run, ctx, cf, torch, reps=20):
    """CheckFree+ keeps replicas of the embedding and de-embedding on the neighbouring stages; a replica
    stays current only if it is copied again every iteration.  Time of one refresh of E + E^-1 (two
    32000 x 2048 fp32 tables), as one call and as k slices issued back to back on the same stream."""
    wl = run.wl
    src_t = list(wl.extra[:2])
    dst_t = [torch.empty_like(t) for t in src_t]
    src, dst = cf.Stage(ctx, src_t), cf.Stage(ctx, dst_t)
    stream = torch.cuda.current_stream()
    n = src.num_chunks
    out = {"bytes_moved": 2 * src.nbytes, "chunks": n}

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

    ms = timed(lambda: cf.cf_copy_stage(ctx, src, dst, stream))
    out["whole_ms"] = round(ms, 5)
    out["whole_GBps"] = round(2 * src.nbytes / ms / 1e6, 1)
    for k in (4, 16, 64):
        per = -(-n // k)
        pieces = [(lo, min(per, n - lo)) for lo in range(0, n, per)]

        def sliced():
            for lo, cnt in pieces:
                cf.cf_copy_stage_range(ctx, src, dst, lo, cnt, stream)
        ms = timed(sliced)
        out[f"in_{len(pieces)}_slices_ms"] = round(ms, 5)
    return out


_ceiling_lib = None


def size_sweep(ctx, cf, torch, sizes_mib=(4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048)):
    """How the three streaming kernels ramp up with the stage size: one flat tensor per stage, buffer
    sets rotated so that every launch finds its data outside the last-level cache (at least 1 GiB is
    cycled through), best of three timed series of back-to-back launches (dispatch gaps included)."""
    import math
    dev = ctx.device
    stream = torch.cuda.current_stream()
    weights = torch.tensor([1.5, 2.5], dtype=torch.float64, device=dev)
    omega = torch.zeros(1, dtype=torch.float64, device=dev)
    rows = []
    for mib in sizes_mib:
        nbytes = mib << 20
        n_sets = max(1, math.ceil((1 << 30) / (3 * nbytes)))
        row = {"MiB_per_stream": mib, "buffer_sets_rotated": n_sets}
        for what, dtype, streams in (("norm", torch.float32, 1), ("blend_fp32", torch.float32, 3),
                                     ("blend_bf16", torch.bfloat16, 3), ("copy", torch.float32, 2)):
            n = nbytes // (2 if dtype == torch.bfloat16 else 4)
            sets = [[torch.empty(n, dtype=torch.float32, device=dev).normal_(0, 1e-2).to(dtype) for _ in range(3)]
                    for _ in range(n_sets)]
            stages = [[cf.Stage(ctx, [t]) for t in st] for st in sets]

            def launch(k):
                a, b, o = stages[k % n_sets]
                if what == "norm":
                    cf.cf_stage_grad_sqnorm(ctx, [a], omega, stream)
                elif what == "copy":
                    cf.cf_copy_stage(ctx, a, o, stream)
                else:
                    cf.cf_recover_stage_weighted_avg(ctx, a, b, weights[0:1], weights[1:2], o, stream)

            reps = max(20, min(2000, int(0.03 / (3 * nbytes / 6.5e12))))
            best = float("inf")
            for _ in range(3):
                for k in range(max(10, reps // 5)):
                    launch(k)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for k in range(reps):
                    launch(k)
                e1.record(stream)
                e1.synchronize()
                best = min(best, e0.elapsed_time(e1) / reps)
            row[what] = {"us": round(best * 1e3, 2), "GBps": round(streams * nbytes / (best * 1e-3) / 1e9, 1)}
            del sets, stages
        rows.append(row)
    return {"what": "bandwidth over stage size (algorithmic bytes / time per call; norm = both passes of one stage)",
            "rows": rows}


def ceiling_library():
    global _ceiling_lib
    if _ceiling_lib is None:
        path = os.path.join(ROOT, "paper_2506_15461_amd", "libcf_ceiling.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is not built; run `python paper_2506_15461_amd/build.py`")
        lib = ctypes.CDLL(path)
        vp = ctypes.c_void_p
        lib.cfc_read.restype = ctypes.c_int
        lib.cfc_read.argtypes = [vp, ctypes.c_uint64, vp, ctypes.c_uint32, vp]
        lib.cfc_copy.restype = ctypes.c_int
        lib.cfc_copy.argtypes = [vp, vp, ctypes.c_uint64, vp]
        _ceiling_lib = lib
    return _ceiling_lib


def measure_ceilings(args, run, ctx, cf, torch, reps=20):
    """What this GPU sustains on one stage's worth of bytes, outside the timed region.  The two
    `trivial_*` figures come from kernels that know nothing of this library (one flat buffer, no chunk
    table, no reduction: csrc/ceiling_kernels.hip); the two `library_*` figures are this library's norm
    (both passes) and copy on the stage's real tensor list; the two `torch_*` figures are PyTorch's own
    device-to-device copies, an outside reference."""
    wl = run.wl
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    src_t = wl.weights[0] + wl.extra if args.config == 4 else wl.weights[wl.lost - 1]
    dst_t = [torch.empty_like(t) for t in src_t]
    src, dst = cf.Stage(ctx, src_t), cf.Stage(ctx, dst_t)
    nbytes = src.nbytes
    omega = torch.zeros(1, dtype=torch.float64, device=ctx.device)

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
    flat_n = nbytes // 16 * 16
    flat_s = torch.empty(flat_n, dtype=torch.uint8, device=ctx.device).random_()
    flat_d = torch.empty_like(flat_s)
    sink = torch.zeros(1, dtype=torch.int32, device=ctx.device)
    lib = ceiling_library()
    num_cu = torch.cuda.get_device_properties(ctx.device).multi_processor_count
    ps, pd, pk = (ctypes.c_void_p(t.data_ptr()) for t in (flat_s, flat_d, sink))
    best = 0.0
    for per_cu in (4, 8, 16):
        ms = timed(lambda: lib.cfc_read(ps, flat_n, pk, num_cu * per_cu, sp))
        best = max(best, flat_n / ms / 1e6)
    out["trivial_read_GBps"] = round(best, 1)
    ms = timed(lambda: lib.cfc_copy(ps, pd, flat_n, sp))
    out["trivial_copy_GBps"] = round(2 * flat_n / ms / 1e6, 1)
    ms = timed(lambda: cf.cf_stage_grad_sqnorm(ctx, [src], omega, stream))
    out["library_norm_GBps"] = round(nbytes / ms / 1e6, 1)
    ms = timed(lambda: cf.cf_copy_stage(ctx, src, dst, stream))
    out["library_copy_GBps"] = round(2 * nbytes / ms / 1e6, 1)
    ms = timed(lambda: torch._foreach_copy_(dst_t, src_t))
    out["torch_foreach_copy_GBps"] = round(2 * nbytes / ms / 1e6, 1)
    ms = timed(lambda: flat_d.copy_(flat_s))
    out["torch_flat_copy_GBps"] = round(2 * flat_n / ms / 1e6, 1)
    out["library_norm_vs_trivial_read"] = round(out["library_norm_GBps"] / out["trivial_read_GBps"], 4)
    out["library_copy_vs_trivial_copy"] = round(out["library_copy_GBps"] / out["trivial_copy_GBps"], 4)
    out["kernels"] = {"trivial_read_GBps": "cfc_read_kernel (best of 4, 8, 16 workgroups per CU)",
                      "trivial_copy_GBps": "cfc_copy_kernel",
                      "library_norm_GBps": "cf_sqnorm_partials_kernel + cf_sqnorm_finalize_kernel",
                      "library_copy_GBps": "cf_copy_kernel",
                      "torch_foreach_copy_GBps": "torch._foreach_copy_", "torch_flat_copy_GBps": "Tensor.copy_"}
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
