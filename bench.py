#!/usr/bin/env python3
"""Benchmark of the fused gradient aggregation + update step on one MI355X.

One "step" = one cmn_allreduce_step call: pack + ring-order K-way sum + scale +
unpack + MomentumSGD over the whole parameter list, gradients already resident in
HBM.  Default workload: ResNet-50 parameter list (161 tensors, 25,557,032 fp32
parameters), K = 32 replicas, 32 ring chunks (the configuration the headline
metric is quoted on).  Prints ONE JSON line on stdout; progress goes to stderr.

  python bench.py [--gpus 1] [--steps 50] [--warmup 5] [--config 3] [--staged] [--no-cpu]
                  [--mean-dest 0|1|2] [--opt sgd|adam] [--grad-dtype ...] [--buckets G] [--overlap]

What the line holds beyond the contract fields:
  roofline.achieved / frac   algorithmic bytes / (time between one pair of HIP events around all timed steps on the
                             launch stream / steps), steps back to back ("warm": parameters and optimizer state of
                             a small model stay in the 256 MB memory-side cache from one step to the next)
  roofline.cold              the same with a 1 GiB read-only sweep between steps (outside the event pairs),
                             so that parameters and state come from HBM as they do after a backward pass
  roofline.copy_ceiling_GBps / read_ceiling_GBps   the best of torch's own copy-like (copy_, add out of place;
                             1 GiB) and read-only (sum, row sums; 4 GiB) kernels, timed by the same event code on
                             the same box: ceilings this library did not write
  roofline.traffic           HBM bytes per step from committed rocprofv3 counter summaries (profiles/),
                             only when workload, options and launched kernel are the profiled ones
  parity_checked             one step from fresh state compared bit for bit with the CPU oracle's
  cpu_baseline               the oracle timed on the host, all cores and one core
"""
import argparse
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak
DT_CODE = {"f32": 0, "f16": 1, "bf16": 2, "i8s": 3}


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
        "adam": 28 * N,
    }[entry]


def step_kernel_name(grad_dtype, kind, mean_dest, opt):
    """Name of the kernel instance a fused step launches, as rocprofv3 prints it (template arguments:
    storage type, loads in flight, [gradient source,] mean destination, optimizer; kind as reported by
    cmn_plan_range_kernel_kind)."""
    dt, o = DT_CODE[grad_dtype], int(opt == "adam")
    return {1: f"k_step<{dt},16,0,{mean_dest},{o}>", 2: f"k_step_two_phase<{dt},8,{mean_dest},{o}>",
            3: f"k_step_state_first<16,{mean_dest},{o}>"}[kind]


def profiled_traffic(workload, kernel, launches_per_step, profiles_dir=None):
    """HBM bytes per step that a committed rocprofv3 counter summary holds for exactly this workload and
    kernel, or (None, None).  Summaries carry one line per measured case:
        TRAFFIC workload=<name> kernel=<instance> launches_per_step=<n> bytes_per_step=<int>"""
    for path in sorted(glob.glob(os.path.join(profiles_dir or os.path.join(ROOT, "profiles"), "*pmc*.txt"))):
        with open(path) as f:
            for line in f:
                if not line.startswith("TRAFFIC "):
                    continue
                kv = dict(x.split("=", 1) for x in line.split()[1:])
                if (kv.get("workload") == workload and kv.get("kernel") == kernel
                        and int(kv.get("launches_per_step", -1)) == launches_per_step):
                    return int(kv["bytes_per_step"]), os.path.relpath(path, ROOT)
    return None, None


def time_launches(torch, fn, steps, warmup, before=None):
    """Per-launch durations (ms) from event pairs on the launch stream, plus wall ms for all.
    `before` runs ahead of every launch, outside its event pair."""
    for _ in range(warmup):
        if before:
            before()
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        if before:
            before()
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [a.elapsed_time(b) for a, b in ev]
    span_ms = ev[0][0].elapsed_time(ev[-1][1])
    return per, span_ms, wall_ms


def time_region(torch, fn, n, warmup):
    """n calls back to back between ONE pair of events on the launch stream (and a synchronize on both sides):
    returns (ms between the events, host wall ms).  An event pair around every single call stretches the period
    between calls by about 7 us on this stack (555 vs 547 us per step on the headline workload) although each
    interval itself reads the same, so whole-region throughput is timed without them."""
    for _ in range(warmup):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b), (time.perf_counter() - t0) * 1e3


def layer_groups(c, n_groups):
    """Cut the tensor list into about equal-sized layer groups, returned last group first
    (the order a backward pass produces gradients in)."""
    edges, acc = [0], 0
    for t, n in enumerate(c.numel):
        acc += n
        if acc >= c.N * len(edges) / n_groups and len(edges) < n_groups:
            edges.append(t + 1)
    edges.append(len(c.numel))
    return [(a, b) for a, b in zip(edges[:-1], edges[1:]) if b > a][::-1]


def measure_overlap(torch, np, c, make_step_range, groups_list, grids, backward_ms, op="mm2048"):
    """Layer-group steps on a second stream while a stand-in backward pass runs on the first.

    The stand-in is a chain of fp32 matmuls (compute-bound, like convolution backward) cut into as many
    slices as there are layer groups; after slice i an event marks group i's gradients as produced, and
    the aggregation stream (same priority) waits for that event before it steps the group.  Reported per
    group count and per width of the step kernels' grid (0: the library's own choice; n: the persistent
    two-phase kernel capped at n workgroups, CMN_TWO_PHASE_GRID): the backward pass alone, the steps alone,
    both overlapped (start of backward to the end of the last step), and the exposed time = overlapped -
    backward alone."""
    side = torch.cuda.Stream()
    shapes = {"mm2048": ((2048, 2048), torch.float32), "mm8192": ((8192, 8192), torch.float32),
              "bmm1024": ((16, 1024, 1024), torch.float32), "mm4096bf16": ((4096, 4096), torch.bfloat16)}
    shape, dt = shapes[op]
    a = torch.randn(*shape, device="cuda").to(dt)
    b = (torch.randn(*shape, device="cuda") * 0.01).to(dt)
    out = torch.empty_like(a)
    mm = torch.bmm if len(shape) == 3 else torch.mm
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        mm(a, b, out=out)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(20):
        mm(a, b, out=out)
    ev1.record()
    torch.cuda.synchronize()
    mm_ms = ev0.elapsed_time(ev1) / 20
    n_mm = max(1, int(round(backward_ms / mm_ms)))
    log(f"[bench] overlap: one {op} = {mm_ms * 1e3:.0f} us; backward stand-in = {n_mm} of them")
    rows = []
    main = torch.cuda.current_stream()

    def timed(run, reps=5):
        times = []
        for _ in range(reps + 1):
            torch.cuda.synchronize()
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record(main)
            run()
            e.record(main)
            torch.cuda.synchronize()
            times.append(s.elapsed_time(e))
        return float(np.median(times[1:]))

    for grid in grids:
        step_range = make_step_range(grid)
        for G in groups_list:
            groups = layer_groups(c, G)
            per_slice = [n_mm // len(groups) + (1 if i < n_mm % len(groups) else 0) for i in range(len(groups))]

            def backward(events=None):
                for i, n in enumerate(per_slice):
                    for _ in range(n):
                        mm(a, b, out=out)
                    if events is not None:
                        events[i].record(main)

            def steps_on(stream, events=None):
                for i, (t0, t1) in enumerate(groups):
                    if events is not None:
                        stream.wait_event(events[i])
                    step_range(t0, t1, stream)

            def both():
                evs = [torch.cuda.Event() for _ in groups]
                side.wait_stream(main)
                backward(evs)
                steps_on(side, evs)
                main.wait_stream(side)          # the end event on `main` then covers both streams

            t_back = timed(lambda: backward())
            t_steps = timed(lambda: steps_on(main))
            t_both = timed(both)
            rows.append({"grid": grid, "layer_groups": len(groups), "backward_alone_us": round(t_back * 1e3, 1),
                         "steps_alone_us": round(t_steps * 1e3, 1), "overlapped_us": round(t_both * 1e3, 1),
                         "exposed_us": round((t_both - t_back) * 1e3, 1),
                         "sequential_us": round((t_back + t_steps) * 1e3, 1)})
            log(f"[bench] overlap grid={grid} G={len(groups)}: backward {t_back * 1e3:.0f} us, steps alone "
                f"{t_steps * 1e3:.0f} us, overlapped {t_both * 1e3:.0f} us -> exposed {(t_both - t_back) * 1e3:.0f} us "
                f"(sequential {(t_back + t_steps) * 1e3:.0f} us)")
    return {"backward_stand_in": f"{n_mm} x torch {op}, {mm_ms * 1e3:.0f} us each", "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = headline)")
    ap.add_argument("--staged", action="store_true", help="also time the four staged entry points (the optimizer-only one is cmn_adam with --opt adam)")
    ap.add_argument("--mean-dest", type=int, default=0, choices=(0, 1, 2),
                    help="0: mean gradient not stored; 1: stored once; 2: written back to all K replicas")
    ap.add_argument("--grad-dtype", default=None, choices=("f32", "f16", "bf16", "i8s"),
                    help="override the gradient storage type of the workload (i8s: random int8 + scales)")
    ap.add_argument("--replicas", type=int, default=None, help="override K (ring chunks follow)")
    ap.add_argument("--opt", default="sgd", choices=("sgd", "adam"), help="optimizer fused into the step")
    ap.add_argument("--buckets", type=int, default=1,
                    help="step the list as this many layer groups of about equal size, last group first "
                         "(cmn_allreduce_step_range per group) instead of one call")
    ap.add_argument("--overlap", action="store_true",
                    help="also run layer-group steps on a second stream under a stand-in backward pass")
    ap.add_argument("--overlap-groups", default="1,4,8,16", help="layer-group counts of the overlap runs")
    ap.add_argument("--overlap-grids", default="0", help="grid widths of the overlap runs (0: the library's choice; "
                                                         "n: persistent kernel capped at n workgroups)")
    ap.add_argument("--backward-op", default="mm2048", choices=("mm2048", "mm8192", "bmm1024", "mm4096bf16"),
                    help="the matmul the stand-in backward pass is made of")
    ap.add_argument("--backward-ms", type=float, default=12.0, help="duration of the stand-in backward pass")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle legs (baseline and parity check)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the torch copy / sum ceilings (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build uses exactly one GPU (all K replicas are resident on it); "
            "--gpus must be 1 and no multi-rank launch is supported.")
        sys.exit(2)

    import dataclasses
    import numpy as np
    import torch
    from paper_1710_11351_amd import binding as B
    from paper_1710_11351_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    B.lib()                                         # fail loudly if libcmn.so is missing
    torch.cuda.set_device(0)
    c = wl.config(args.config)
    synthetic_override = False
    if args.grad_dtype and args.grad_dtype != c.grad_dtype:
        c = dataclasses.replace(c, grad_dtype=args.grad_dtype, name=f"{c.name}+{args.grad_dtype}")
        synthetic_override = True
    if args.replicas and args.replicas != c.K:
        c = dataclasses.replace(c, K=args.replicas, n_chunks=args.replicas, name=f"{c.name}+k{args.replicas}")
        synthetic_override = True
    use_cpu = not args.no_cpu and not synthetic_override and c.grad_dtype != "i8s"
    log(f"[bench] workload {c.name}: T={len(c.tensors)} N={c.N} K={c.K} chunks={c.n_chunks} grads={c.grad_dtype}")

    tg = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i8s": torch.int8}[c.grad_dtype]
    t0 = time.time()
    host_grads = []                                 # kept for the CPU legs
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
                if use_cpu:
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
    adam = args.opt == "adam"
    it = [0]
    if adam:
        d_s = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in c.numel]
        plan.bind_adam(d_s)

    def step_range(t0_, t1_, stream=None):
        if adam:
            plan.allreduce_adam_step_range(t0_, t1_, 1e-3, 0.9, 0.999, 1e-8, c.wd, max(1, it[0]), mean_dest=args.mean_dest,
                                           stream=stream)
        else:
            plan.allreduce_step_range(t0_, t1_, c.lr, c.mu, c.wd, mean_dest=args.mean_dest, stream=stream)

    groups = [(0, len(c.numel))] if args.buckets <= 1 else layer_groups(c, args.buckets)
    if args.buckets > 1:
        log(f"[bench] {len(groups)} layer groups, stepped last group first")

    def step():
        it[0] += 1
        for a_, b_ in groups:
            step_range(a_, b_)
    kinds = {B.cmn_plan_range_kernel_kind(plan.h, a_, b_, adam, args.mean_dest) for a_, b_ in groups}
    kernel = "mixed" if len(kinds) > 1 else step_kernel_name(c.grad_dtype, kinds.pop(), args.mean_dest, args.opt)
    # launches per step of the two-phase kernel: one per round of the persistent grid
    torch.cuda.synchronize()

    span_ms, wall_ms = time_region(torch, step, args.steps, args.warmup)
    ms_per_step = span_ms / args.steps              # whole timed region / steps
    kern_ms = ms_per_step                           # average duration of one step's launches, gaps between steps included
    abytes = algorithmic_bytes(c, "step", args.mean_dest, args.opt)
    value = abytes / (ms_per_step * 1e-3) / 1e9
    achieved = abytes / (kern_ms * 1e-3) / 1e9
    per, _, _ = time_launches(torch, step, min(10, args.steps), 0)     # single launches, each under its own pair of events
    log(f"[bench] fused step: {ms_per_step * 1e3:.1f} us/step over {args.steps} steps between one pair of events "
        f"(host wall {wall_ms / args.steps * 1e3:.1f} us; single launches under their own event pairs: mean "
        f"{np.mean(per) * 1e3:.1f} us, min {min(per) * 1e3:.1f} us) "
        f"-> {value:.0f} GB/s effective = {value / HBM_PEAK_GBPS:.3f} of HBM peak")

    # The same launches with the caches swept in between: a read-only pass over 1 GiB (four times the
    # memory-side cache) stands in for the forward and backward passes that separate two steps of a real
    # iteration, so parameters and optimizer state are fetched from HBM.  The sweep is outside the event pairs.
    sweep_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    cold_per, _, _ = time_launches(torch, step, max(10, args.steps // 2), 2, before=lambda: sweep_src.sum())
    cold_ms = float(np.mean(cold_per))
    cold = {"kernel_us": round(cold_ms * 1e3, 2), "achieved": round(abytes / (cold_ms * 1e-3) / 1e9, 1),
            "frac": round(abytes / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "sweep": "torch.sum over 1 GiB fp32 before every step, outside the event pair (every launch under its own pair)"}
    log(f"[bench] fused step after a cache sweep: {cold_ms * 1e3:.1f} us per launch -> {cold['achieved']:.0f} GB/s "
        f"= {cold['frac']:.3f} of HBM peak")
    del sweep_src

    extra = {}
    if args.staged:
        packed = torch.empty(c.K * plan.L, dtype=tg, device="cuda")
        reduced = torch.empty(plan.L, dtype=torch.float32, device="cuda")
        optimizer_only = (("adam", lambda: plan.adam(1e-3, 0.9, 0.999, 1e-8, c.wd, max(1, it[0]))) if adam else
                          ("momentum_sgd", lambda: plan.momentum_sgd(c.lr, c.mu, c.wd)))
        for name, fn in (("pack", lambda: plan.pack(packed)), ("ring_reduce", lambda: plan.ring_reduce(packed, reduced)),
                         ("scale_unpack", lambda: plan.scale_unpack(reduced)), optimizer_only):
            n = max(5, args.steps // 2)
            us = time_region(torch, fn, n, 2)[0] / n * 1e3
            ab = algorithmic_bytes(c, name)
            extra[name] = {"us": round(us, 1), "GBps": round(ab / (us * 1e-6) / 1e9, 1)}
            log(f"[bench] {name}: {extra[name]['us']} us, {extra[name]['GBps']} GB/s effective")
        del packed, reduced

    overlap = None
    if args.overlap:
        narrow = {}

        def make_step_range(grid):
            if grid == 0:
                return step_range
            saved = {k: os.environ.get(k) for k in ("CMN_TWO_PHASE_GRID", "CMN_STEP_KERNEL")}
            os.environ.update(CMN_TWO_PHASE_GRID=str(grid), CMN_STEP_KERNEL="two_phase")   # read at plan creation
            try:
                q = narrow[grid] = B.Plan(c.numel, c.K, c.n_chunks, c.align_bytes, c.grad_dtype)
            finally:
                for k, v in saved.items():
                    os.environ.pop(k, None) if v is None else os.environ.__setitem__(k, v)
            q.bind(d_g, d_p, d_v, d_m)
            if adam:
                q.bind_adam(d_s)
                return lambda t0_, t1_, stream=None: q.allreduce_adam_step_range(
                    t0_, t1_, 1e-3, 0.9, 0.999, 1e-8, c.wd, max(1, it[0]), mean_dest=args.mean_dest, stream=stream)
            return lambda t0_, t1_, stream=None: q.allreduce_step_range(t0_, t1_, c.lr, c.mu, c.wd,
                                                                       mean_dest=args.mean_dest, stream=stream)
        overlap = measure_overlap(torch, np, c, make_step_range, [int(x) for x in args.overlap_groups.split(",")],
                                  [int(x) for x in args.overlap_grids.split(",")], args.backward_ms, args.backward_op)

    # Ceilings of this box from code this library did not write, timed by the same event code.  torch offers no
    # tuned streaming probe, so several of its kernels are tried and the best one of a kind is the ceiling:
    # read only: sum over all of 4 GiB, and row sums of the same buffer viewed as 2^20 x 2^10;
    # read + write: copy_ (the runtime's device copy) and add(x, 1, out=y) (an elementwise kernel) over 1 GiB each.
    # The last figure is the library's own gather kernel used as a 1 GiB -> 1 GiB copy; rocprofv3's FETCH_SIZE /
    # WRITE_SIZE counters are calibrated on it.
    ceil = {}
    if not args.no_ceilings:
        cal_n = 1 << 28
        src = torch.empty(cal_n, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty(cal_n, dtype=torch.float32, device="cuda")
        gbps = lambda nbytes, fn: round(nbytes / (time_region(torch, fn, 10, 2)[0] / 10 * 1e-3) / 1e9, 1)
        ops = {"copy_": gbps(2 * cal_n * 4, lambda: dst.copy_(src)),
               "add_out": gbps(2 * cal_n * 4, lambda: torch.add(src, 1.0, out=dst))}
        cal = B.Plan([cal_n], 1, 1, 256, "f32")
        cal.bind([[src]], None, None, None)
        ceil["device_copy_GBps"] = gbps(2 * cal_n * 4, lambda: cal.pack(dst))
        del dst, cal, src
        big = torch.empty(1 << 30, dtype=torch.float32, device="cuda").normal_()
        ops["sum_all"] = gbps(big.numel() * 4, lambda: big.sum())
        ops["sum_rows"] = gbps(big.numel() * 4, lambda: big.view(1 << 20, 1 << 10).sum(1))
        del big
        ceil = {"copy_ceiling_GBps": max(ops["copy_"], ops["add_out"]), "read_ceiling_GBps": max(ops["sum_all"], ops["sum_rows"]),
                "vendor_ops_GBps": ops, **ceil}
        ceil["frac_of_read_ceiling"] = round(achieved / ceil["read_ceiling_GBps"], 4)
        log(f"[bench] ceilings on this box (torch): read {ceil['read_ceiling_GBps']:.0f} GB/s, read+write "
            f"{ceil['copy_ceiling_GBps']:.0f} GB/s {ops}; cmn_pack as a 1 GiB copy {ceil['device_copy_GBps']:.0f} GB/s")

    cpu, parity = None, None
    if use_cpu and args.opt == "sgd" and args.mean_dest in (0, 1):
        import oracle                                # CPU legs only: baseline timing and the parity check
        threads = oracle.max_threads()
        run = lambda p_o, v_o: oracle.allreduce_step(host_grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd,
                                                     dtype=c.grad_dtype, align_bytes=c.align_bytes)
        times, p_o, v_o = [], None, None
        while len(times) < 3 or (sum(times) < 10.0 and len(times) < 40):   # whole steps, about 10 s of them
            p_o, v_o = [x.copy() for x in p_h], [x.copy() for x in v_h]
            t1 = time.perf_counter()
            mean_o = run(p_o, v_o)
            times.append(time.perf_counter() - t1)
        dt, reps = float(np.mean(times)), len(times)
        oracle.set_threads(1)
        single = []
        for _ in range(2):
            p1, v1 = [x.copy() for x in p_h], [x.copy() for x in v_h]
            t1 = time.perf_counter()
            run(p1, v1)
            single.append(time.perf_counter() - t1)
        oracle.set_threads(threads)
        dt1 = float(np.mean(single))
        cpu = {"value": round(abytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"{reps} full steps of {c.name} (all {c.N} elements, K={c.K}), mean {dt:.2f} s each; "
                         f"OpenMP over ring chunks in the fold, the other steps single-threaded",
               "us_per_step": round(dt * 1e6, 1),
               "single_thread": {"value": round(abytes / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                                 "us_per_step": round(dt1 * 1e6, 1), "sample": "2 full steps of the same workload"}}
        log(f"[bench] CPU oracle: {dt:.2f} s/step on {threads} threads -> {cpu['value']} GB/s effective; "
            f"{dt1:.2f} s/step on one thread -> {cpu['single_thread']['value']} GB/s")
        # Parity of the timed path in this very run: fresh state, one step of the same entry point and kernel,
        # every parameter and velocity (and the mean gradient, if stored) against the oracle's step, bit for bit.
        for d, h in zip(d_p + d_v, p_h + v_h):
            d.copy_(torch.from_numpy(h))
        step()
        torch.cuda.synchronize()
        same = all(np.array_equal(a.view(np.uint32), b.view(np.uint32))
                   for a, b in zip(B.download_tensors(d_p) + B.download_tensors(d_v), p_o + v_o))
        if args.mean_dest == 1:
            same = same and all(np.array_equal(a.view(np.uint32), b.view(np.uint32))
                                for a, b in zip(B.download_tensors(d_m), mean_o))
        parity = bool(same)
        log(f"[bench] one step from fresh state vs the oracle: {'bit-identical' if parity else 'MISMATCH'}")

    n_launch = sum(B.cmn_plan_range_launch_count(plan.h, a_, b_, adam, args.mean_dest) for a_, b_ in groups)
    traffic, traffic_source = (None, None) if args.buckets > 1 else profiled_traffic(c.name, kernel, n_launch)
    out = {
        "metric": "effective HBM GB/s + µs per ResNet-50 allreduce+update step at K=32" if args.config == 3 and not synthetic_override
                  else f"effective HBM GB/s + us per allreduce+update step ({c.name})",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",                              # sums, averages and updates are float32 whatever the storage type
        "storage_dtype": c.grad_dtype, "data": "synthetic",
        "config": {"workload": c.name, "tensors": len(c.tensors), "elements": c.N, "replicas_K": c.K,
                   "ring_chunks": c.n_chunks, "grad_storage": c.grad_dtype, "mean_dest": args.mean_dest,
                   "optimizer": args.opt, "layer_groups": args.buckets,
                   "entry": "cmn_allreduce_adam_step" if adam else "cmn_allreduce_step"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "clock": "one pair of HIP events on the launch stream around all timed steps, divided by the number of "
                              "steps (gaps between steps included; steps back to back, so the state of a small model stays "
                              "in the memory-side cache)",
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel, "launches_per_step": n_launch,
                     "algorithmic_bytes": abytes, "kernel_us": round(kern_ms * 1e3, 2),
                     "single_launch_us": {"mean": round(float(np.mean(per)) * 1e3, 2), "min": round(min(per) * 1e3, 2)},
                     "cold": cold, **ceil},
        "parity_checked": parity,
        "cpu_baseline": cpu,
    }
    if extra:
        out["staged"] = extra
    if overlap:
        out["overlap"] = overlap
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
