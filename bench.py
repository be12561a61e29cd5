#!/usr/bin/env python3
"""Benchmark of the fused gradient aggregation + update step on one MI355X.

One "step" = one cmn_allreduce_step launch: pack + ring-order K-way sum + scale +
unpack + MomentumSGD over the whole parameter list, gradients already resident in
HBM.  Default workload: ResNet-50 parameter list (161 tensors, 25,557,032 fp32
parameters), K = 32 replicas, 32 ring chunks (the configuration the headline
metric is quoted on).  Prints ONE JSON line on stdout; progress goes to stderr.

  python bench.py [--gpus 1] [--steps 50] [--warmup 5] [--config 3] [--staged] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak

# HBM bytes per launch of the fused kernel at config 3 read by rocprofv3 --pmc
# (FETCH_SIZE, WRITE_SIZE), scaled by the same counters' reading of a plain copy of
# known size (scale 2.0 for FETCH_SIZE, 1.0 for WRITE_SIZE).  Source: profiles/allreduce_step_resnet50_k32_pmc.txt
MEASURED_TRAFFIC_BYTES = {3: 3_691_800_000}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(c, entry="step", mean_dest=0, opt="sgd"):
    """Bytes the method must move per launch (padding, tables, scratch not counted)."""
    eg = {"f32": 4, "f16": 2, "bf16": 2, "i8s": 1}[c.grad_dtype]
    N, K = c.N, c.K
    state = 24 if opt == "adam" else 16                         # p + optimizer state, read and written
    mean = {0: 0, 1: 4, 2: K * eg}[mean_dest]                   # averaged gradient written once / K times
    return {
        "step": (K * eg + state + mean) * N,
        "pack": 2 * K * eg * N,
        "ring_reduce": (K * eg + 4) * N,
        "scale_unpack": 8 * N,
        "momentum_sgd": 20 * N,
    }[entry]


def time_launches(torch, fn, steps, warmup):
    """Per-launch durations (ms) from event pairs on the launch stream, plus wall ms for all."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [a.elapsed_time(b) for a, b in ev]
    span_ms = ev[0][0].elapsed_time(ev[-1][1])
    return per, span_ms, wall_ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = headline)")
    ap.add_argument("--staged", action="store_true", help="also time the four staged entry points")
    ap.add_argument("--mean-dest", type=int, default=0, choices=(0, 1, 2),
                    help="0: mean gradient not stored; 1: stored once; 2: written back to all K replicas")
    ap.add_argument("--grad-dtype", default=None, choices=("f32", "f16", "bf16", "i8s"),
                    help="override the gradient storage type of the workload (i8s: random int8 + scales)")
    ap.add_argument("--opt", default="sgd", choices=("sgd", "adam"), help="optimizer fused into the step")
    ap.add_argument("--buckets", type=int, default=1,
                    help="step the list as this many layer groups of about equal size, last group first "
                         "(cmn_allreduce_step_range per group) instead of one call")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build uses exactly one GPU (all K replicas are resident on it); "
            "--gpus must be 1 and no multi-rank launch is supported.")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1710_11351_amd import binding as B
    from paper_1710_11351_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    B.lib()                                         # fail loudly if libcmn.so is missing
    torch.cuda.set_device(0)
    c = wl.config(args.config)
    if args.grad_dtype and args.grad_dtype != c.grad_dtype:
        import dataclasses
        c = dataclasses.replace(c, grad_dtype=args.grad_dtype, name=f"{c.name}+{args.grad_dtype}")
        args.no_cpu = True
    log(f"[bench] workload {c.name}: T={len(c.tensors)} N={c.N} K={c.K} chunks={c.n_chunks} grads={c.grad_dtype}")

    tg = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i8s": torch.int8}[c.grad_dtype]
    t0 = time.time()
    host_grads = []                                 # kept for the CPU leg when it fits
    keep_host = not args.no_cpu
    d_g = []
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=8) as ex:   # numpy's generators release the GIL
        for k0 in range(0, c.K, 8):
            if c.grad_dtype == "i8s":               # timing only: random int8 payload, scales bound below
                batch = [[torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda") for n in c.numel]
                         for _ in range(k0, min(c.K, k0 + 8))]
            else:
                batch = list(ex.map(lambda k: wl.gen_grads(c, 0, k), range(k0, min(c.K, k0 + 8))))
            for g in batch:
                if c.grad_dtype == "i8s":
                    d_g.append(g)
                elif c.grad_dtype == "bf16":
                    d_g.append([torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).cuda() for h in g])
                else:
                    d_g.append(B.upload_tensors(g))     # every tensor its own allocation
                if keep_host:
                    host_grads.append(g)
            log(f"[bench] generated + uploaded replicas {len(d_g)}/{c.K} ({time.time() - t0:.1f}s)")
    p_h, v_h = wl.gen_params(c), wl.gen_velocity(c)
    d_p, d_v = B.upload_tensors(p_h), B.upload_tensors(v_h)
    d_m = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in c.numel]
    plan = B.Plan(c.numel, c.K, c.n_chunks, c.align_bytes, c.grad_dtype)
    plan.bind(d_g, d_p, d_v, d_m)
    if c.grad_dtype == "i8s":
        d_sc = [torch.rand(c.n_chunks, device="cuda") * 1e-5 + 1e-6 for _ in range(c.K)]
        plan.bind_scales(d_sc)
    if args.opt == "adam":
        d_s = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in c.numel]
        plan.bind_adam(d_s)
        it = [0]

        def step():
            it[0] += 1
            plan.allreduce_adam_step(1e-3, 0.9, 0.999, 1e-8, c.wd, it[0], mean_dest=args.mean_dest)
    else:
        step = lambda: plan.allreduce_step(c.lr, c.mu, c.wd, mean_dest=args.mean_dest)
    if args.buckets > 1:                            # layer groups of about N / buckets elements, back to front
        edges, acc = [0], 0
        for t, n in enumerate(c.numel):
            acc += n
            if acc >= c.N * len(edges) / args.buckets and len(edges) < args.buckets:
                edges.append(t + 1)
        edges.append(len(c.numel))
        groups = [(a, b) for a, b in zip(edges[:-1], edges[1:]) if b > a][::-1]
        log(f"[bench] {len(groups)} layer groups, stepped last group first")
        if args.opt == "adam":
            def step():
                it[0] += 1
                for a, b in groups:
                    plan.allreduce_adam_step_range(a, b, 1e-3, 0.9, 0.999, 1e-8, c.wd, it[0], mean_dest=args.mean_dest)
        else:
            def step():
                for a, b in groups:
                    plan.allreduce_step_range(a, b, c.lr, c.mu, c.wd, mean_dest=args.mean_dest)
    torch.cuda.synchronize()

    per, span_ms, wall_ms = time_launches(torch, step, args.steps, args.warmup)
    ms_per_step = span_ms / args.steps              # whole timed region / steps
    kern_ms = float(np.mean(per))                   # average duration of one launch
    abytes = algorithmic_bytes(c, "step", args.mean_dest, args.opt)
    value = abytes / (ms_per_step * 1e-3) / 1e9
    achieved = abytes / (kern_ms * 1e-3) / 1e9
    log(f"[bench] fused step: {ms_per_step * 1e3:.1f} us/step over {args.steps} steps "
        f"(per-launch mean {kern_ms * 1e3:.1f} us, min {min(per) * 1e3:.1f} us, host wall {wall_ms / args.steps * 1e3:.1f} us) "
        f"-> {value:.0f} GB/s effective = {value / HBM_PEAK_GBPS:.3f} of HBM peak")

    extra = {}
    if args.staged:
        packed = torch.empty(c.K * plan.L, dtype=tg, device="cuda")
        reduced = torch.empty(plan.L, dtype=torch.float32, device="cuda")
        for name, fn in (("pack", lambda: plan.pack(packed)), ("ring_reduce", lambda: plan.ring_reduce(packed, reduced)),
                         ("scale_unpack", lambda: plan.scale_unpack(reduced)),
                         ("momentum_sgd", lambda: plan.momentum_sgd(c.lr, c.mu, c.wd))):
            pr, sp, _ = time_launches(torch, fn, max(5, args.steps // 2), 2)
            ab = algorithmic_bytes(c, name)
            extra[name] = {"us": round(float(np.mean(pr)) * 1e3, 1), "GBps": round(ab / (np.mean(pr) * 1e-3) / 1e9, 1)}
            log(f"[bench] {name}: {extra[name]['us']} us, {extra[name]['GBps']} GB/s effective")
        del packed, reduced

    # A plain copy of known size through the library's own gather kernel (one tensor,
    # one replica: cmn_pack degenerates to a 1 GiB -> 1 GiB copy).  It gives the box's
    # copy rate as context and calibrates the rocprofv3 FETCH_SIZE / WRITE_SIZE counters.
    cal_n = 1 << 28
    src = torch.empty(cal_n, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty(cal_n, dtype=torch.float32, device="cuda")
    cal = B.Plan([cal_n], 1, 1, 256, "f32")
    cal.bind([[src]], None, None, None)
    pr, _, _ = time_launches(torch, lambda: cal.pack(dst), 10, 2)
    copy_gbps = 2 * cal_n * 4 / (float(np.mean(pr)) * 1e-3) / 1e9
    log(f"[bench] calibration copy (cmn_pack, 1 GiB -> 1 GiB): {copy_gbps:.0f} GB/s (read+write)")
    del src, dst, cal

    cpu = None
    if not args.no_cpu and (args.opt, args.mean_dest) == ("sgd", 0):
        import oracle                                # CPU baseline leg only
        threads = oracle.max_threads()
        times = []
        while len(times) < 3 or (sum(times) < 10.0 and len(times) < 40):   # whole steps, about 10 s of them
            p_o, v_o = [x.copy() for x in p_h], [x.copy() for x in v_h]
            t1 = time.perf_counter()
            oracle.allreduce_step(host_grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd, dtype=c.grad_dtype,
                                  align_bytes=c.align_bytes)
            times.append(time.perf_counter() - t1)
        dt, reps = float(np.mean(times)), len(times)
        cpu = {"value": round(abytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"{reps} full steps of {c.name} (all {c.N} elements, K={c.K}), mean {dt:.2f} s each; "
                         f"OpenMP over ring chunks in the fold, the other steps single-threaded",
               "us_per_step": round(dt * 1e6, 1)}
        log(f"[bench] CPU oracle: {dt:.2f} s/step on {threads} threads -> {cpu['value']} GB/s effective")

    traffic = MEASURED_TRAFFIC_BYTES.get(args.config) if (args.opt, args.mean_dest, args.buckets) == ("sgd", 0, 1) else None
    out = {
        "metric": "effective HBM GB/s + \u00b5s per ResNet-50 allreduce+update step at K=32" if args.config == 3
                  else f"effective HBM GB/s + us per allreduce+update step ({c.name})",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": c.name, "tensors": len(c.tensors), "elements": c.N, "replicas_K": c.K,
                   "ring_chunks": c.n_chunks, "grad_storage": c.grad_dtype, "mean_dest": args.mean_dest,
                   "optimizer": args.opt, "layer_groups": args.buckets,
                   "entry": "cmn_allreduce_adam_step" if args.opt == "adam" else "cmn_allreduce_step"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": "k_step_two_phase" if B.cmn_plan_step_kernel_kind(plan.h, args.opt == "adam", args.mean_dest) == 2
                               else "k_step",
                     "algorithmic_bytes": abytes,
                     "kernel_us": round(kern_ms * 1e3, 2), "device_copy_GBps": round(copy_gbps, 1)},
        "cpu_baseline": cpu,
    }
    if extra:
        out["staged"] = extra
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
