"""Shared driver of the GPU parity tests: runs the oracle and the HIP path on the
same seeded host arrays and compares every output the path produces."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
from paper_1710_11351_amd import binding as B
from paper_1710_11351_amd import workloads as wl


def bits(a):
    a = np.ascontiguousarray(a)
    if a.dtype in (np.uint16, np.int8):
        return a
    return a.view(np.uint16 if a.dtype == np.float16 else np.uint32)


def assert_bit_equal(got, want, what):
    got, want = np.asarray(got).reshape(-1), np.asarray(want).reshape(-1)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    bad = np.nonzero(bits(got) != bits(want))[0]
    if bad.size:
        both_nan = np.isnan(got[bad]) & np.isnan(want[bad])
        bad = bad[~both_nan]
    assert bad.size == 0, (f"{what}: {bad.size} of {got.size} elements differ, first at {bad[:5]}: "
                           f"got {got[bad[:5]]} want {want[bad[:5]]}")


def assert_update_close(got, want, what, rel=1e-6):
    """The stated bar for the optimizer outputs: |a-b| <= rel * max(|b|, rms(b)) per tensor."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    if want.size == 0:
        return
    rms = np.sqrt(np.mean(want ** 2))
    err = np.abs(got - want) - rel * np.maximum(np.abs(want), rms)
    assert np.all(err <= 0), f"{what}: exceeds {rel} relative by {err.max()}"


def to_numpy(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DeviceCase:
    """Device tensors of one workload, each tensor its own allocation.  misalign: every tensor starts
    that many elements past its allocation; a tuple (even replicas, odd replicas, parameters and
    optimizer state, mean gradient) gives each group its own offset, so that the streams of a tile
    share no 16-byte alignment and the kernels fall back to their element-by-element path."""

    def __init__(self, c: wl.Config, ring_rotate=1, misalign=0, with_mean=True, adam=False):
        import torch
        self.c, self.torch = c, torch
        tg = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i8s": torch.int8}[c.grad_dtype]
        self.plan = B.Plan(c.numel, c.K, c.n_chunks, c.align_bytes, c.grad_dtype, ring_rotate)

        mis = misalign if isinstance(misalign, tuple) else (misalign,) * 4

        def alloc(dtype, off):
            out = []
            for n in c.numel:
                buf = torch.zeros(n + off, dtype=dtype, device="cuda")
                out.append(buf[off:])
            return out

        self.grads = [alloc(tg, mis[k % 2]) for k in range(c.K)]
        self.p, self.v = alloc(torch.float32, mis[2]), alloc(torch.float32, mis[2])
        self.m = alloc(torch.float32, mis[3]) if with_mean else None
        self.plan.bind(self.grads, self.p, self.v, self.m)
        self.scales = None
        if c.grad_dtype == "i8s":
            self.scales = [torch.ones(c.n_chunks, dtype=torch.float32, device="cuda") for _ in range(c.K)]
            self.plan.bind_scales(self.scales)
        self.s = None
        if adam:
            self.s = alloc(torch.float32, mis[2])
            self.plan.bind_adam(self.s)

    def set_state(self, p_host, v_host):
        for d, h in zip(self.p, p_host):
            d.copy_(self.torch.from_numpy(h))
        for d, h in zip(self.v, v_host):
            d.copy_(self.torch.from_numpy(h))

    def set_grads(self, k, g_host):
        for d, h in zip(self.grads[k], g_host):
            h = np.ascontiguousarray(h)
            if h.dtype == np.uint16:                       # bfloat16 bit patterns
                d.copy_(self.torch.from_numpy(h.view(np.int16)).view(self.torch.bfloat16))
            else:
                d.copy_(self.torch.from_numpy(h))

    def set_scales(self, k, s_host):
        self.scales[k].copy_(self.torch.from_numpy(np.ascontiguousarray(s_host, dtype=np.float32)))

    def get(self, tensors):
        self.torch.cuda.synchronize()
        return [to_numpy(t) for t in tensors]


def gen_all_grads(c: wl.Config, step: int, unquantised=False):
    """All K replicas' gradients of one iteration (numpy's generators release the GIL)."""
    fn = wl.gen_grads_f32_unquantised if unquantised else wl.gen_grads
    if c.K * c.N < 4_000_000:
        return [fn(c, step, k) for k in range(c.K)]
    with ThreadPoolExecutor(max_workers=8) as ex:
        return list(ex.map(lambda k: fn(c, step, k), range(c.K)))


ADAM = dict(alpha=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)     # the optimizer's published defaults


def run_parity(c: wl.Config, steps=3, ring_rotate=1, misalign=0, staged=True, fused=True, check_packed=True,
               opt="sgd", bucketed=False):
    """Oracle vs HIP on `steps` consecutive iterations with fresh gradients each.
    opt: "sgd" (MomentumSGD) or "adam"; bucketed: run the fused step as per-layer-group
    range calls, last group first, instead of one call."""
    import torch
    adam = opt == "adam"
    p_o = [x.copy() for x in wl.gen_params(c)]
    v_o = [x.copy() for x in wl.gen_velocity(c)]
    s_o = [x.copy() for x in wl.gen_velocity(c)]            # Adam's second moments start at zero too
    cases = {}
    if fused:
        cases["fused"] = DeviceCase(c, ring_rotate, misalign, adam=adam)
    if staged:
        cases["staged"] = DeviceCase(c, ring_rotate, misalign, adam=adam)
    for dc in cases.values():
        dc.set_state(p_o, v_o)
    geo = oracle.Geometry(c.numel, c.n_chunks, c.align_bytes, c.grad_dtype)
    if staged:
        dc = cases["staged"]
        tg = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i8s": torch.int8}[c.grad_dtype]
        packed = torch.full((c.K * geo.L + 64,), 7, dtype=tg, device="cuda")[: c.K * geo.L]
        reduced = torch.full((geo.L + 64,), 7.0, dtype=torch.float32, device="cuda")[: geo.L]
        assert dc.plan.L == geo.L

    for step in range(steps):
        grads = gen_all_grads(c, step)
        scales = None
        if c.grad_dtype == "i8s":                      # producer-side quantisation of the f32 draws
            qs = [wl.quantise_i8(g, geo.chunk_elems, geo.C) for g in grads]
            grads, scales = [q for q, _ in qs], [s for _, s in qs]
        print(f"[parity] {c.name} step {step}: inputs ready", flush=True)
        for dc in cases.values():
            for k in range(c.K):
                dc.set_grads(k, grads[k])
                if scales is not None:
                    dc.set_scales(k, scales[k])
        # ---- oracle, step by step with intermediates
        packed_o = [oracle.pack(geo, grads[k]) for k in range(c.K)]
        total_o = oracle.direct_fold(geo, packed_o, ring_rotate, scales)
        mean_o = oracle.unpack(geo, oracle.scale(total_o, c.K))
        for t in range(geo.T):
            if adam:
                oracle.adam(mean_o[t], p_o[t], v_o[t], s_o[t], ADAM["alpha"], ADAM["beta1"], ADAM["beta2"],
                            ADAM["eps"], c.wd, step + 1)
            else:
                oracle.momentum_sgd(mean_o[t], p_o[t], v_o[t], c.lr, c.mu, c.wd)

        if staged:
            dc = cases["staged"]
            dc.plan.pack(packed)
            if check_packed and (step == 0 or c.K * geo.L < 50_000_000):
                torch.cuda.synchronize()
                for k in range(c.K):
                    assert_bit_equal(to_numpy(packed[k * geo.L:(k + 1) * geo.L]), packed_o[k],
                                     f"step {step} packed[{k}]")
            dc.plan.ring_reduce(packed, reduced)
            torch.cuda.synchronize()
            assert_bit_equal(reduced.cpu().numpy(), total_o, f"step {step} ring_reduce")
            dc.plan.scale_unpack(reduced)
            for t, (a, b) in enumerate(zip(dc.get(dc.m), mean_o)):
                assert_bit_equal(a, b, f"step {step} staged mean_grad[{t}]")
            if adam:
                dc.plan.adam(ADAM["alpha"], ADAM["beta1"], ADAM["beta2"], ADAM["eps"], c.wd, step + 1)
            else:
                dc.plan.momentum_sgd(c.lr, c.mu, c.wd)
            _compare_state(dc, p_o, v_o, f"step {step} staged", s_o if adam else None)
        if fused:
            dc = cases["fused"]
            write_mean = step % 2 == 0
            if write_mean:
                for m in dc.m:
                    m.fill_(-5.0)
            groups = [(0, geo.T)]
            if bucketed:                                    # uneven layer groups, output layer first
                cuts = sorted({0, geo.T, geo.T // 7, geo.T // 3, geo.T // 2, geo.T - 1} & set(range(geo.T + 1)))
                groups = list(zip(cuts[:-1], cuts[1:]))[::-1] + [(geo.T, geo.T)]
            for t0, t1 in groups:
                if adam:
                    dc.plan.allreduce_adam_step_range(t0, t1, ADAM["alpha"], ADAM["beta1"], ADAM["beta2"], ADAM["eps"],
                                                      c.wd, step + 1, mean_dest=int(write_mean))
                else:
                    dc.plan.allreduce_step_range(t0, t1, c.lr, c.mu, c.wd, mean_dest=int(write_mean))
            _compare_state(dc, p_o, v_o, f"step {step} fused", s_o if adam else None)
            if write_mean:
                for t, (a, b) in enumerate(zip(dc.get(dc.m), mean_o)):
                    assert_bit_equal(a, b, f"step {step} fused mean_grad[{t}]")
        del packed_o, total_o
    return p_o, v_o


def _compare_state(dc, p_o, v_o, what, s_o=None):
    if s_o is not None:
        for t, (a, b) in enumerate(zip(dc.get(dc.s), s_o)):
            assert_update_close(a, b, f"{what} second moment[{t}]")
            assert_bit_equal(a, b, f"{what} second moment[{t}]")
    for t, (a, b) in enumerate(zip(dc.get(dc.p), p_o)):
        assert_update_close(a, b, f"{what} p[{t}]")     # the stated bar
        assert_bit_equal(a, b, f"{what} p[{t}]")        # what the kernels actually achieve
    for t, (a, b) in enumerate(zip(dc.get(dc.v), v_o)):
        assert_update_close(a, b, f"{what} v[{t}]")
        assert_bit_equal(a, b, f"{what} v[{t}]")
