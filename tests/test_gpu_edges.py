"""Edge values, overlapped launches and binding rules of the HIP path against the CPU oracle (needs the GPU)."""
import numpy as np
import pytest

import oracle
from paper_1710_11351_amd import binding as B
from paper_1710_11351_amd import workloads as wl
from parity_util import DeviceCase, assert_bit_equal, gen_all_grads

pytestmark = pytest.mark.gpu

F32_MAX = np.float32(3.4028235e38)


def _special_grads(dtype, K, numel, rng):
    """K replicas' gradient tensors in the storage type, ordinary draws with IEEE edge values planted at
    fixed positions of every tensor: infinities of both signs, NaN, signed zeros, the largest finite value
    (twice: the float32 sum of two bfloat16 / float32 maxima overflows), the smallest subnormals.  For int8
    storage the edge cases are in the scales (returned second; None otherwise)."""
    if dtype == "i8s":
        q = [[rng.integers(-128, 128, n, dtype=np.int8) for n in numel] for _ in range(K)]
        for k in range(K):
            for t in q[k]:
                if t.size >= 8:
                    t[:8] = [-128, 127, 0, -1, 1, 127, -128, 0]
        return q, None
    edge32 = np.array([np.inf, -np.inf, np.nan, -0.0, 0.0, F32_MAX, F32_MAX, -F32_MAX, 1e-45, -1e-45, 1.1754942e-38, 65504.0,
                       -65504.0, 5.9604645e-08, 6.1035156e-05, 1.0], np.float32)
    out = []
    for k in range(K):
        row = []
        for n in numel:
            x = (rng.standard_normal(n) * 1e-2).astype(np.float32)
            m = min(n, edge32.size)
            # replica k plants the edge values rotated by k, so that an element sees inf + finite, inf - inf,
            # max + max, subnormal + subnormal, -0 + -0 ... across the replicas
            x[:m] = np.roll(edge32, k if k < 3 else 0)[:m]
            if n > 40:
                x[32:40] = [-0.0] * 8                    # every replica: the sum of negative zeros keeps its sign
            if dtype == "f16":
                with np.errstate(over="ignore"):
                    x = x.astype(np.float16)             # max float32 becomes inf, 1e-45 becomes 0: still edge values
            elif dtype == "bf16":
                bits = (x.view(np.uint32) >> 16).astype(np.uint16)        # truncation: exact for these edge values
                bits[np.isnan(x)] = 0x7FC0
                x = bits
            row.append(x)
        out.append(row)
    return out, None


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8s"])
@pytest.mark.parametrize("K", [2, 9])
@pytest.mark.parametrize("path", ["fused", "staged"])
def test_special_values_through_every_storage_type(dtype, K, path):
    """Inf, NaN, signed zeros, subnormals, largest finite values and (int8) degenerate scales travel through
    decode, the fixed-order sum, the scale and the update exactly as the oracle's plain float32 arithmetic says
    (every worker obtains the same average, also when it is Inf or NaN)."""
    import torch
    numel = [40, 3, 2100, 0, 1024, 5000]
    c = wl.custom_config(numel, K=K, n_chunks=3, grad_dtype=dtype, cfg=58, wd=1e-3)
    rng = np.random.default_rng(58 + K)
    grads, _ = _special_grads(dtype, K, numel, rng)
    geo = oracle.Geometry(numel, c.n_chunks, 256, dtype)
    scales = None
    if dtype == "i8s":                                   # chunk 0: products overflow; chunk 1: Inf; chunk 2: NaN
        scales = [np.full(geo.C, 1e-3 * (k + 1), np.float32) for k in range(K)]
        scales[0][:] = [1e-3, np.inf, np.nan]
        scales[1][:] = [3e38, 1e-45, -0.0]
    dc = DeviceCase(c)
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], [x.copy() for x in wl.gen_velocity(c)]
    dc.set_state(p_o, v_o)
    for k in range(K):
        dc.set_grads(k, grads[k])
        if scales is not None:
            dc.set_scales(k, scales[k])
    packed_o = [oracle.pack(geo, grads[k]) for k in range(K)]
    with np.errstate(all="ignore"):
        total_o = oracle.direct_fold(geo, packed_o, 1, scales)
        mean_o = oracle.unpack(geo, oracle.scale(total_o, K))
        for t in range(geo.T):
            oracle.momentum_sgd(mean_o[t], p_o[t], v_o[t], c.lr, c.mu, c.wd)
    flat = np.concatenate(mean_o)
    assert np.isnan(flat).any() and np.isinf(flat).any()        # the edge values really reach the result
    if path == "fused":
        dc.plan.allreduce_step(c.lr, c.mu, c.wd, write_mean_grad=True)
    else:
        tg = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i8s": torch.int8}[dtype]
        packed = torch.empty(K * geo.L, dtype=tg, device="cuda")
        reduced = torch.empty(geo.L, dtype=torch.float32, device="cuda")
        dc.plan.pack(packed)
        dc.plan.ring_reduce(packed, reduced)
        torch.cuda.synchronize()
        assert_bit_equal(reduced.cpu().numpy(), total_o, "ring_reduce")
        dc.plan.scale_unpack(reduced)
        dc.plan.momentum_sgd(c.lr, c.mu, c.wd)
    for name, dev, ref in (("mean", dc.m, mean_o), ("p", dc.p, p_o), ("v", dc.v, v_o)):
        for t, (a, b) in enumerate(zip(dc.get(dev), ref)):
            assert_bit_equal(a, b, f"{path} {name}[{t}]")


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("K", [2, 8])
def test_average_handed_back_is_rounded_like_the_oracle_at_ties_and_edges(dtype, K):
    """All-replica mode encodes the float32 average on the device: ties go to even, the largest finite value
    stays finite, subnormal results are kept, NaN stays NaN, Inf stays Inf, -0 stays -0."""
    numel = [4096 + 64, 40]
    c = wl.custom_config(numel, K=K, n_chunks=2, grad_dtype=dtype, cfg=57)
    one = {"f16": np.float32(2.0 ** -10), "bf16": np.float32(2.0 ** -7), "f32": np.float32(2.0 ** -23)}[dtype]   # ulp of 1.0
    mx = {"f16": np.float32(65504.0), "bf16": np.float32(3.3895314e38), "f32": F32_MAX}[dtype]
    tiny = {"f16": np.float32(2.0 ** -24), "bf16": np.float32(2.0 ** -133), "f32": np.float32(1e-45)}[dtype]
    # (value held by replica 0, value held by every other replica)
    cases = [(1.0, 1.0 + one), (1.0 + one, 1.0 + 2 * one), (1.0 + one, 1.0), (mx, mx), (-mx, -mx), (tiny, 0.0), (tiny, tiny),
             (3 * tiny, 0.0), (np.inf, 1.0), (np.inf, -np.inf), (np.nan, 1.0), (-0.0, -0.0), (0.0, -0.0), (-tiny, 0.0),
             (mx, mx - mx * one), (6.1035156e-05, 6.1035156e-05 - 2.0 ** -24)]
    grads = []
    for k in range(K):
        row = []
        for n in numel:
            x = np.full(n, 0.25, np.float32)
            for i, (a, b) in enumerate(cases):
                x[i::64] = a if k == 0 else b          # every 64th slot: all vector lanes and the ragged tail
            with np.errstate(over="ignore"):
                row.append(x.astype(np.float16) if dtype == "f16" else
                           oracle.float_to_bf16(x) if dtype == "bf16" else x)
        grads.append(row)
    dc = DeviceCase(c)
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], wl.gen_velocity(c)
    dc.set_state(p_o, v_o)
    for k in range(K):
        dc.set_grads(k, grads[k])
    with np.errstate(all="ignore"):
        mean_o = oracle.allreduce_step(grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd, dtype=dtype)
        want = [{"f16": oracle.float_to_half, "bf16": oracle.float_to_bf16, "f32": lambda x: x}[dtype](m) for m in mean_o]
    dc.plan.allreduce_step(c.lr, c.mu, c.wd, mean_dest=B.CMN_MEAN_TO_ALL_REPLICAS)
    for k in range(K):
        for t, (a, b) in enumerate(zip(dc.get(dc.grads[k]), want)):
            assert_bit_equal(a, b, f"replica {k} tensor {t}")
    for t, (a, b) in enumerate(zip(dc.get(dc.p) + dc.get(dc.v), p_o + v_o)):
        assert_bit_equal(a, b, f"state {t}")


@pytest.mark.parametrize("K", [4, 9])
def test_layer_groups_stepped_on_a_second_stream_as_their_gradients_arrive(K):
    """The overlap pattern of a training loop: stream A "produces" the gradients of one layer group after the
    other (last group first) and records an event after each; stream B waits for that event and steps the
    group.  The result must be the oracle's, whatever the interleaving."""
    import torch
    numel = [4096, 64, 64, 36864, 256, 256, 9408, 1000, 147456, 512]
    c = wl.custom_config(numel, K=K, n_chunks=4, cfg=56, wd=1e-3)
    dc = DeviceCase(c)
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], wl.gen_velocity(c)
    dc.set_state(p_o, v_o)
    groups = [(8, 10), (5, 8), (3, 5), (0, 3)]
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    for step in range(3):
        grads = gen_all_grads(c, step)
        staged = [[torch.from_numpy(g).cuda() for g in row] for row in grads]      # what the backward pass will produce
        torch.cuda.synchronize()
        events = []
        with torch.cuda.stream(a):
            for t0, t1 in groups:
                for k in range(K):
                    for t in range(t0, t1):
                        dc.grads[k][t].copy_(staged[k][t], non_blocking=True)
                ev = torch.cuda.Event()
                ev.record(a)
                events.append(ev)
        for (t0, t1), ev in zip(groups, events):
            b.wait_event(ev)
            dc.plan.allreduce_step_range(t0, t1, c.lr, c.mu, c.wd, stream=b)
        oracle.allreduce_step(grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd)
        a.synchronize(); b.synchronize()
        for t, (x, y) in enumerate(zip(dc.get(dc.p) + dc.get(dc.v), p_o + v_o)):
            assert_bit_equal(x, y, f"step {step} state {t}")
        a.wait_stream(b)                                   # the next iteration's gradients must not overtake this step


def test_a_new_binding_drops_adam_moments_and_int8_scales():
    """cmn_plan_bind starts afresh: second moments and scales bound before it must be bound again."""
    c = wl.custom_config([1000, 24], K=2, n_chunks=2, cfg=55)
    dc = DeviceCase(c, adam=True)
    adam = lambda: B.cmn_allreduce_adam_step(dc.plan.h, 1e-3, .9, .999, 1e-8, 0., 1, 0)
    assert adam() == B.CMN_OK
    dc.plan.bind(dc.grads, dc.p, dc.v, dc.m)
    assert adam() == B.CMN_EUNBOUND and B.cmn_adam(dc.plan.h, 1e-3, .9, .999, 1e-8, 0., 1) == B.CMN_EUNBOUND
    assert B.cmn_allreduce_step(dc.plan.h, .1, .9, 0., 0) == B.CMN_OK          # MomentumSGD needs no second moments
    dc.plan.bind_adam(dc.s)
    assert adam() == B.CMN_OK
    c8 = wl.custom_config([1000, 24], K=2, n_chunks=2, grad_dtype="i8s", cfg=55)
    d8 = DeviceCase(c8)
    assert B.cmn_allreduce_step(d8.plan.h, .1, .9, 0., 0) == B.CMN_OK
    d8.plan.bind(d8.grads, d8.p, d8.v, d8.m)
    assert B.cmn_allreduce_step(d8.plan.h, .1, .9, 0., 0) == B.CMN_EUNBOUND
    d8.plan.bind_scales(d8.scales)
    assert B.cmn_allreduce_step(d8.plan.h, .1, .9, 0., 0) == B.CMN_OK
    import torch
    torch.cuda.synchronize()


def test_config3_resnet50_k32_every_chunk_folded_from_rank_0_full_size():
    """The other reading of "ring reduction in rank order" (ring_rotate = 0) on the benchmark workload."""
    from parity_util import run_parity
    run_parity(wl.config(3), steps=1, ring_rotate=0)


# ---- the widened variants bench.py times and profiles/ records, at the benchmark's full size ----
@pytest.mark.parametrize("dtype", ["bf16", "i8s"])
def test_config3_resnet50_k32_compressed_storage_full_size(dtype):
    """ResNet-50 x 32 replicas with bfloat16 (two-phase kernel) and int8 + per-chunk scales (one-pass kernel)."""
    import dataclasses
    from parity_util import run_parity
    c = dataclasses.replace(wl.config(3), grad_dtype=dtype, name=f"resnet50_k32_{dtype}")
    run_parity(c, steps=1, check_packed=False)


def test_config3_resnet50_k32_average_to_all_replicas_full_size():
    """The all-gather half on the benchmark workload: all 32 replicas' 161 tensors end up holding the average."""
    c = wl.config(3)
    dc = DeviceCase(c, with_mean=False)
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], wl.gen_velocity(c)
    dc.set_state(p_o, v_o)
    grads = gen_all_grads(c, 0)
    for k in range(c.K):
        dc.set_grads(k, grads[k])
    mean_o = oracle.allreduce_step(grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd)
    del grads
    dc.plan.allreduce_step(c.lr, c.mu, c.wd, mean_dest=B.CMN_MEAN_TO_ALL_REPLICAS)
    for k in range(c.K):
        for t, (a, b) in enumerate(zip(dc.get(dc.grads[k]), mean_o)):
            assert_bit_equal(a, b, f"replica {k} tensor {t}")
    for t, (a, b) in enumerate(zip(dc.get(dc.p) + dc.get(dc.v), p_o + v_o)):
        assert_bit_equal(a, b, f"state {t}")


def test_bench_line_carries_the_contract_fields_and_its_own_parity_check(step_kernel_mode):
    """bench.py on the small workload: one JSON line on stdout with the contract's fields, the roofline and
    cpu_baseline objects, and a parity check of the timed entry point against the oracle that came out true."""
    if step_kernel_mode != "auto":
        pytest.skip("the benchmark is run once, with the library's own kernel choice")
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--config", "1", "--steps", "5", "--warmup", "2"],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "parity_checked"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["unit"] == "GB/s" and d["dtype"] == "f32" and d["vs_baseline"] is None
    assert d["config"]["workload"] == "mlp_k2_f32" and d["parity_checked"] is True
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert rf["kernel"] == "k_step_state_first<16,0,0>" and rf["launches_per_step"] == 1 and "traffic" in rf
    assert rf["cold"]["kernel_us"] > 0 and rf["read_ceiling_GBps"] > 1000 and rf["copy_ceiling_GBps"] > 1000
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["single_thread"]["cores"] == 1
