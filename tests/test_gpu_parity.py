"""HIP path vs CPU oracle, element by element, through the C-ABI (needs the GPU)."""
import numpy as np
import pytest

from paper_1710_11351_amd import workloads as wl
from parity_util import run_parity

pytestmark = pytest.mark.gpu


def test_config1_mlp_k2():
    run_parity(wl.config(1), steps=3)


@pytest.mark.parametrize("rot", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8s"])
def test_ragged_list_with_empty_tensors(dtype, rot):
    # odd sizes, empty tensors, tiles and vectors that straddle tensor and chunk edges, K not a power of two
    numel = [5, 0, 5000, 1, 64, 12345, 7, 0, 2049, 3]
    c = wl.custom_config(numel, K=3, n_chunks=5, grad_dtype=dtype, cfg=91, wd=1e-3,
                         outlier_frac=0.01 if dtype == "f16" else 0.0)
    run_parity(c, steps=3, ring_rotate=rot)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i8s"])
@pytest.mark.parametrize("misalign", [1, 3])
def test_unaligned_base_pointers(dtype, misalign):
    c = wl.custom_config([1000, 4096, 37, 8192 + 5], K=4, n_chunks=4, grad_dtype=dtype, cfg=92)
    run_parity(c, steps=2, misalign=misalign)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("misalign", [0, 1, 3])
def test_ragged_unaligned_lists_with_ten_replicas(dtype, misalign):
    numel = [5, 0, 5000, 1, 64, 12345, 7, 0, 2049, 3, 70000]
    c = wl.custom_config(numel, K=10, n_chunks=7, grad_dtype=dtype, cfg=77, wd=1e-3)
    run_parity(c, steps=2, misalign=misalign)


@pytest.mark.parametrize("env", [{"CMN_STEP_KERNEL": "stream"}, {"CMN_STEP_KERNEL": "two_phase", "CMN_TWO_PHASE_GRID": "2"}])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_launch_shape_knobs_do_not_change_results(monkeypatch, env, dtype):
    """The two environment knobs read at plan creation pick another kernel or grid size; the result
    stays the oracle's, bit for bit (also under a forced kernel kind)."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    numel = [5, 0, 5000, 1, 64, 12345, 7, 2049, 3, 30000]
    c = wl.custom_config(numel, K=12, n_chunks=6, grad_dtype=dtype, cfg=76, wd=1e-3)
    run_parity(c, steps=2, misalign=1)
    run_parity(c, steps=1, staged=True, fused=False)


@pytest.mark.parametrize("dtype,opt", [("f32", "sgd"), ("f16", "sgd"), ("f32", "adam"), ("bf16", "adam")])
def test_two_phase_rounds_at_small_size(monkeypatch, dtype, opt):
    """Three persistent workgroups instead of two per compute unit: the list no longer fits one
    round of the register stash, so the one-launch-per-round split (fused step and ring reduce)
    is exercised at a size the oracle finishes quickly."""
    monkeypatch.setenv("CMN_TWO_PHASE_GRID", "3")
    numel = [200_000, 5, 0, 150_001, 64, 70_000, 7, 2049]
    c = wl.custom_config(numel, K=8, n_chunks=5, grad_dtype=dtype, cfg=75, wd=1e-3)
    run_parity(c, steps=2, misalign=0, opt=opt)
    run_parity(c, steps=1, misalign=1, opt=opt, staged=False)


@pytest.mark.parametrize("K", [3, 9])                 # a few and several replicas (either kernel kind is also forced, see conftest.py)
@pytest.mark.parametrize("dtype,opt", [("f32", "sgd"), ("f16", "sgd"), ("bf16", "adam"), ("f32", "adam")])
@pytest.mark.parametrize("mis", [(1, 1, 2, 2), (0, 1, 0, 0), (0, 0, 0, 1), (2, 2, 1, 3)])
def test_streams_without_a_common_alignment(K, dtype, opt, mis):
    """Gradients, parameters/state and mean gradient start at different offsets from a 16-byte
    boundary (or the replicas disagree among themselves): some or all kernel variants find no
    common alignment and must process whole tiles element by element, with the same bits."""
    numel = [5, 3000, 0, 1025, 64, 4099]
    c = wl.custom_config(numel, K=K, n_chunks=4, grad_dtype=dtype, cfg=74, wd=1e-3)
    run_parity(c, steps=2, misalign=mis, opt=opt)


def _random_case(seed):
    rng = np.random.default_rng(seed)
    sizes = [0, 1, 3, 7, 8, 63, 64, 1000, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 5000, 12345, 40000]
    numel = [int(rng.choice(sizes)) for _ in range(int(rng.integers(1, 10)))]
    if sum(numel) == 0:
        numel.append(777)
    dtype = str(rng.choice(["f32", "f32", "f16", "bf16", "i8s"]))
    mis = int(rng.integers(0, 4))
    misalign = mis if rng.random() < 0.7 else tuple(int(x) for x in rng.integers(0, 4, size=4))
    return dict(numel=numel, K=int(rng.integers(1, 21)), C=int(rng.integers(1, 10)), dtype=dtype, misalign=misalign,
                opt=str(rng.choice(["sgd", "adam"])), rot=int(rng.integers(0, 2)), wd=float(rng.choice([0.0, 1e-3])),
                bucketed=bool(rng.random() < 0.3))


@pytest.mark.parametrize("seed", range(20))
def test_random_lists_replica_counts_and_alignments(seed):
    """Seeded random workloads: list shapes around the tile sizes, 1..20 replicas, 1..9 ring chunks,
    every storage type, common and conflicting misalignments, both optimizers, both fold orders."""
    k = _random_case(seed)
    c = wl.custom_config(k["numel"], K=k["K"], n_chunks=k["C"], grad_dtype=k["dtype"], cfg=60 + seed, wd=k["wd"],
                         outlier_frac=0.01 if k["dtype"] == "f16" else 0.0)
    run_parity(c, steps=2, ring_rotate=k["rot"], misalign=k["misalign"], opt=k["opt"], staged=not k["bucketed"],
               bucketed=k["bucketed"])


def test_single_replica_is_the_plain_optimizer():
    c = wl.custom_config([3000, 100], K=1, n_chunks=1, cfg=93)
    run_parity(c, steps=2)


def test_fewer_elements_than_chunks():
    c = wl.custom_config([3, 2], K=4, n_chunks=8, cfg=94)     # most chunks are pure padding
    run_parity(c, steps=2)


def test_more_chunks_than_replicas_and_k7():
    c = wl.custom_config([70000, 333], K=7, n_chunks=14, cfg=95)
    run_parity(c, steps=2)


def test_many_replicas_f16_k40():
    c = wl.custom_config([20000, 1000, 24], K=40, n_chunks=40, grad_dtype="f16", cfg=96, outlier_frac=0.01)
    run_parity(c, steps=2)


def test_bf16_storage_adam_k33():
    c = wl.custom_config([20000, 1000, 24, 4096], K=33, n_chunks=11, grad_dtype="bf16", cfg=86)
    run_parity(c, steps=2, opt="adam")


def test_int8_storage_adam_and_many_chunks():
    c = wl.custom_config([70000, 333, 4096, 5], K=9, n_chunks=18, grad_dtype="i8s", cfg=81, wd=1e-3)
    run_parity(c, steps=2, opt="adam")


def test_int8_storage_error_bound_and_argument_checks():
    """Quantising with scale = max|g|/127 per chunk moves an element by at most scale/2 (plus one fp32
    rounding of q*scale), so the mean moves by at most mean_k(scale_k)/2 * (1 + 2^-22)."""
    import torch
    import oracle
    from paper_1710_11351_amd import binding as B
    from parity_util import DeviceCase, gen_all_grads
    numel = [36864, 64, 147456, 1000]
    c = wl.custom_config(numel, K=8, n_chunks=8, grad_dtype="i8s", cfg=80, grad_std=1e-3)
    dc = DeviceCase(c)
    geo = oracle.Geometry(numel, c.n_chunks, 256, "i8s")
    assert B.cmn_allreduce_step(dc.plan.h, c.lr, c.mu, 0., B.CMN_MEAN_TO_ALL_REPLICAS) == B.CMN_EINVAL
    g32 = gen_all_grads(c, 0)
    qs = [wl.quantise_i8(g, geo.chunk_elems, geo.C) for g in g32]
    for k, (q, s) in enumerate(qs):
        dc.set_grads(k, q); dc.set_scales(k, s)
    dc.set_state(wl.gen_params(c), wl.gen_velocity(c))
    dc.plan.allreduce_step(c.lr, c.mu, c.wd, write_mean_grad=True)
    got = np.concatenate(dc.get(dc.m)).astype(np.float64)
    want = np.mean(np.stack([np.concatenate(g).astype(np.float64) for g in g32]), axis=0)
    half_step = np.mean(np.stack([s for _, s in qs]).astype(np.float64), axis=0) / 2          # per chunk
    bound = np.repeat(half_step, geo.chunk_elems)[:want.size] * (1 + 2.0 ** -22) + 1e-12
    assert np.all(np.abs(got - want) <= bound)
    assert np.max(np.abs(got - want)) > 0.05 * bound.max()      # the quantisation error is really there
    # a CMN_I8S plan without scales refuses to run
    p2 = B.Plan(numel, c.K, c.n_chunks, 256, "i8s")
    p2.bind(dc.grads, dc.p, dc.v, dc.m)
    assert B.cmn_allreduce_step(p2.h, c.lr, c.mu, 0., 0) == B.CMN_EUNBOUND
    assert B.cmn_ring_reduce(p2.h, 256, 512) == B.CMN_EUNBOUND
    assert B.cmn_plan_bind_scales(dc.plan.h, None) == B.CMN_ENULL
    pf = B.Plan(numel, 2, 2)
    assert B.cmn_plan_bind_scales(pf.h, [256, 512]) == B.CMN_EINVAL             # not an int8 plan


def test_bf16_storage_within_8e3_of_unquantised_fp32():
    """bfloat16 keeps 8 significant bits: rounding moves an element by at most 2^-9 = 1.95e-3 of its
    magnitude, so the mean moves by at most 1.95e-3 * mean_k |g_k|; asserted with the bar 8e-3 / 2 = 4e-3."""
    import torch
    from paper_1710_11351_amd import binding as B
    from parity_util import gen_all_grads, to_numpy
    numel = [36864, 64, 147456, 1000]
    c = wl.custom_config(numel, K=16, n_chunks=16, grad_dtype="bf16", cfg=85, grad_std=1e-3)
    gq = gen_all_grads(c, 0)
    g32 = gen_all_grads(c, 0, unquantised=True)
    d_g = [[torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).cuda() for h in g] for g in gq]
    d_p = B.upload_tensors(wl.gen_params(c)); d_v = B.upload_tensors(wl.gen_velocity(c))
    d_m = [torch.zeros(n, device="cuda") for n in numel]
    plan = B.Plan(numel, c.K, c.n_chunks, 256, "bf16")
    plan.bind(d_g, d_p, d_v, d_m)
    plan.allreduce_step(c.lr, c.mu, c.wd, write_mean_grad=True)
    got = B.download_tensors(d_m)
    for t in range(len(numel)):
        st = np.stack([g[t].astype(np.float64) for g in g32])
        want, mag = st.mean(axis=0), np.abs(st).mean(axis=0)
        assert np.all(np.abs(got[t] - want) <= 4e-3 * np.maximum(np.abs(want), mag)), f"tensor {t}"
        assert np.max(np.abs(got[t] - want)) > 0


@pytest.mark.parametrize("K", [2, 8])             # a few and several replicas (either kernel kind is also forced, see conftest.py)
def test_special_values_propagate(K):
    import torch
    from paper_1710_11351_amd import binding as B
    n = 1024
    plan = B.Plan([n], K, 2)
    a = np.zeros(n, np.float32); b = np.zeros(n, np.float32)
    a[0], b[0] = np.inf, 1.0
    a[1], b[1] = np.inf, -np.inf
    a[2], b[2] = -0.0, -0.0
    a[3], b[3] = 1e-45, 1e-45
    a[4], b[4] = 1e-40, 2e-40
    rest = np.zeros(n, np.float32); rest[2] = -0.0                      # the other K-2 replicas add nothing
    g = [[torch.from_numpy(a).cuda()], [torch.from_numpy(b).cuda()]] + [[torch.from_numpy(rest).cuda()] for _ in range(K - 2)]
    p = [torch.zeros(n, device="cuda")]; v = [torch.zeros(n, device="cuda")]; m = [torch.ones(n, device="cuda")]
    plan.bind(g, p, v, m)
    plan.allreduce_step(1.0, 0.0, 0.0, write_mean_grad=True)
    out = m[0].cpu().numpy()
    s = np.float32(1.0) / np.float32(K)
    assert out[0] == np.inf and np.isnan(out[1])
    assert out[2] == 0 and np.signbit(out[2])
    assert out[3] == (np.float32(1e-45) + np.float32(1e-45)) * s         # subnormals are kept, not flushed
    assert out[4] == (np.float32(1e-40) + np.float32(2e-40)) * s and out[4] != 0
    assert not out[5:].any()
    pv = p[0].cpu().numpy()
    assert pv[0] == -np.inf and np.isnan(pv[1])                           # and reach the parameters


def test_empty_plan_is_a_no_op():
    from paper_1710_11351_amd import binding as B
    plan = B.Plan([0, 0], 2, 2)
    import torch
    e = lambda: [torch.zeros(0, device="cuda") for _ in range(2)]
    plan.bind([e(), e()], e(), e(), e())
    plan.pack(None); plan.ring_reduce(None, None); plan.scale_unpack(None)
    plan.momentum_sgd(.1, .9, 0.); plan.allreduce_step(.1, .9, 0., True)
    torch.cuda.synchronize()


def test_config2_resnet50_k4_full_size():
    run_parity(wl.config(2), steps=3)


# ---- widened rows: bucketed (per layer group) steps, Adam, average handed back to every replica ----
@pytest.mark.parametrize("K", [5, 8])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("opt", ["sgd", "adam"])
def test_bucketed_range_steps_equal_one_full_step(dtype, opt, K):
    numel = [5, 0, 5000, 1, 64, 12345, 7, 0, 2049, 3, 800, 4096]
    c = wl.custom_config(numel, K=K, n_chunks=5, grad_dtype=dtype, cfg=98, wd=1e-3)
    run_parity(c, steps=2, staged=False, opt=opt, bucketed=True)


@pytest.mark.parametrize("K", [6, 12])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("misalign", [0, 3])
def test_adam_fused_and_staged(dtype, misalign, K):
    numel = [1000, 4096, 37, 8192 + 5, 0, 64]
    c = wl.custom_config(numel, K=K, n_chunks=3, grad_dtype=dtype, cfg=99, wd=5e-4 if misalign else 0.0)
    run_parity(c, steps=3, opt="adam", misalign=misalign)


def test_range_arguments_are_validated():
    from paper_1710_11351_amd import binding as B
    from parity_util import DeviceCase
    dc = DeviceCase(wl.custom_config([100, 200, 300], K=2, n_chunks=2, cfg=89))
    for t0, t1 in ((-1, 2), (2, 1), (0, 4)):
        assert B.cmn_allreduce_step_range(dc.plan.h, t0, t1, .1, .9, 0., 0) == B.CMN_EINVAL
    assert B.cmn_allreduce_step(dc.plan.h, .1, .9, 0., 3) == B.CMN_EINVAL              # unknown destination
    assert B.cmn_allreduce_adam_step(dc.plan.h, 1e-3, .9, .999, 1e-8, 0., 1, 0) == B.CMN_EUNBOUND   # no second moments
    assert B.cmn_allreduce_step_range(dc.plan.h, 1, 1, .1, .9, 0., 0) == B.CMN_OK      # empty range: no-op


@pytest.mark.parametrize("K", [5, 9])             # a few and several replicas (either kernel kind is also forced, see conftest.py)
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("misalign", [0, 1])
def test_average_is_handed_back_to_every_replica(dtype, misalign, K):
    """The all-gather half of the allreduce: afterwards every worker's gradient tensors hold the
    average (rounded to nearest even when the workers store binary16)."""
    import oracle
    from paper_1710_11351_amd import binding as B
    from parity_util import DeviceCase, assert_bit_equal, gen_all_grads
    numel = [3000, 0, 77, 4096, 1, 2050]
    c = wl.custom_config(numel, K=K, n_chunks=4, grad_dtype=dtype, cfg=88, outlier_frac=0.01 if dtype == "f16" else 0.0)
    dc = DeviceCase(c, misalign=misalign)
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], wl.gen_velocity(c)
    dc.set_state(p_o, v_o)
    for step in range(2):
        grads = gen_all_grads(c, step)
        for k in range(c.K):
            dc.set_grads(k, grads[k])
        mean_o = oracle.allreduce_step(grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd, dtype=dtype)
        dc.plan.allreduce_step(c.lr, c.mu, c.wd, mean_dest=B.CMN_MEAN_TO_ALL_REPLICAS)
        want = [{"f16": oracle.float_to_half, "bf16": oracle.float_to_bf16, "f32": lambda x: x}[dtype](m) for m in mean_o]
        for k in range(c.K):
            for t, (a, b) in enumerate(zip(dc.get(dc.grads[k]), want)):
                assert_bit_equal(a, b, f"step {step} replica {k} tensor {t}")
        for t, (a, b) in enumerate(zip(dc.get(dc.p) + dc.get(dc.v), p_o + v_o)):
            assert_bit_equal(a, b, f"step {step} state {t}")


@pytest.mark.parametrize("K", [3, 9])             # a few and several replicas (either kernel kind is also forced, see conftest.py)
@pytest.mark.parametrize("staged", [False, True])
def test_mean_gradient_may_overwrite_replica_0(K, staged):
    """The mean-gradient tensors may be replica 0's own float32 gradient tensors: every kernel
    has read an element's K gradients before it writes the element's average."""
    import oracle
    import torch
    from parity_util import DeviceCase, assert_bit_equal, gen_all_grads
    numel = [3000, 0, 77, 4096, 1, 2050]
    c = wl.custom_config(numel, K=K, n_chunks=4, cfg=73, wd=1e-3)
    dc = DeviceCase(c, misalign=1)
    dc.plan.bind(dc.grads, dc.p, dc.v, dc.grads[0])
    p_o, v_o = [x.copy() for x in wl.gen_params(c)], wl.gen_velocity(c)
    dc.set_state(p_o, v_o)
    for step in range(2):
        grads = gen_all_grads(c, step)
        for k in range(c.K):
            dc.set_grads(k, grads[k])
        mean_o = oracle.allreduce_step(grads, p_o, v_o, c.n_chunks, c.lr, c.mu, c.wd)
        if staged:
            packed = torch.empty(c.K * dc.plan.L, dtype=torch.float32, device="cuda")
            reduced = torch.empty(dc.plan.L, dtype=torch.float32, device="cuda")
            dc.plan.pack(packed); dc.plan.ring_reduce(packed, reduced); dc.plan.scale_unpack(reduced)
            dc.plan.momentum_sgd(c.lr, c.mu, c.wd)
        else:
            dc.plan.allreduce_step(c.lr, c.mu, c.wd, write_mean_grad=True)
        for t, (a, b) in enumerate(zip(dc.get(dc.grads[0]) + dc.get(dc.p) + dc.get(dc.v), mean_o + p_o + v_o)):
            assert_bit_equal(a, b, f"step {step} tensor {t}")


# ---- the benchmark workloads at full size, in the launch configuration bench.py times ----
def test_config3_resnet50_k32_full_size():
    run_parity(wl.config(3), steps=3)


def test_config4_resnet50_k128_f16_full_size():
    run_parity(wl.config(4), steps=2)


def test_config5_vgg16_k16_weight_decay_full_size():
    run_parity(wl.config(5), steps=2)


def test_config5_vgg16_k16_adam_staged_full_size():
    """The optimizer-only kernels on a model larger than the memory-side cache (streaming loads and stores)."""
    run_parity(wl.config(5), steps=1, opt="adam", fused=False)


def test_more_than_2_to_31_elements_full_size(monkeypatch):
    """One tensor of 2^31 + 5000 binary16 elements (offsets beyond 32 bits in every kernel), two replicas.
    The oracle cannot hold this whole, so every element is checked against the same arithmetic written with
    torch's elementwise fp32 operations, each of which rounds once: (g0 + g1) * 0.5, mu*v - lr*g, p + v; and the
    oracle itself is run on windows of the big tensor (its start, the elements around packed index 2^31, around
    the ring-chunk edge, its tail) and on the two small tensors.  With two replicas the fold is one addition,
    which commutes, so a window's result does not depend on where the window lies."""
    import torch
    import oracle
    from paper_1710_11351_amd import binding as B
    from parity_util import assert_bit_equal
    n = (1 << 31) + 5000
    numel = [777, n, 3]
    gen = torch.Generator(device="cuda").manual_seed(4242)
    def rnd(m, dt, std):
        out = torch.empty(m, dtype=dt, device="cuda")
        for a in range(0, m, 1 << 28):                      # generated piecewise to bound the temporaries
            b = min(m, a + (1 << 28))
            out[a:b] = (torch.randn(b - a, device="cuda", generator=gen) * std).to(dt)
        return out
    g = [[rnd(m, torch.float16, 1e-2) for m in numel] for _ in range(2)]
    p = [rnd(m, torch.float32, 0.05) for m in numel]
    v = [rnd(m, torch.float32, 0.01) for m in numel]
    m_fused = [torch.empty(m, dtype=torch.float32, device="cuda") for m in numel]
    lr, mu = 0.1, 0.9
    want_p, want_v, want_m = [], [], []
    for t in range(len(numel)):
        mean = (g[0][t].float() + g[1][t].float()) * 0.5
        nv = mu * v[t] - lr * mean
        want_m.append(mean); want_v.append(nv); want_p.append(p[t] + nv)
    plan = B.Plan(numel, 2, 2, 256, "f16")
    edge, at31 = plan.chunk_elems - numel[0], (1 << 31) - numel[0]       # tensor coordinates of the chunk edge / packed 2^31
    windows = [(0, 0, numel[0]), (2, 0, numel[2]), (1, 0, 4096), (1, at31 - 2048, at31 + 2048),
               (1, edge - 2048, edge + 2048), (1, n - 4096, n)]
    p_host = {w: p[w[0]][w[1]:w[2]].cpu().numpy() for w in windows}       # state before any step
    v_host = {w: v[w[0]][w[1]:w[2]].cpu().numpy() for w in windows}

    def oracle_windows(what, got_m, got_p=None, got_v=None):
        for w in windows:
            t, lo, hi = w
            geo = oracle.Geometry([hi - lo], 1, 256, "f16")
            packed_o = [oracle.pack(geo, [g[k][t][lo:hi].cpu().numpy()]) for k in range(2)]
            mean_o = oracle.unpack(geo, oracle.scale(oracle.direct_fold(geo, packed_o, 1), 2))[0]
            assert_bit_equal(got_m[t][lo:hi].cpu().numpy(), mean_o, f"{what} mean, window {w}")
            if got_p is not None:
                p_o, v_o = p_host[w].copy(), v_host[w].copy()
                oracle.momentum_sgd(mean_o, p_o, v_o, lr, mu, 0.0)
                assert_bit_equal(got_p[t][lo:hi].cpu().numpy(), p_o, f"{what} p, window {w}")
                assert_bit_equal(got_v[t][lo:hi].cpu().numpy(), v_o, f"{what} v, window {w}")
    # staged entry points first (they leave p and v untouched until cmn_momentum_sgd, which is skipped)
    plan.bind(g, p, v, m_fused)
    packed = torch.empty(2 * plan.L, dtype=torch.float16, device="cuda")
    reduced = torch.empty(plan.L, dtype=torch.float32, device="cuda")
    plan.pack(packed); plan.ring_reduce(packed, reduced); plan.scale_unpack(reduced)
    torch.cuda.synchronize()
    oracle_windows("staged", m_fused)
    for t in range(len(numel)):
        assert torch.equal(m_fused[t].view(torch.int32), want_m[t].view(torch.int32)), f"staged mean, tensor {t}"
        m_fused[t].zero_()
    del packed, reduced, plan
    p0, v0 = [x.clone() for x in p], [x.clone() for x in v]
    for mode in ("stream", "two_phase"):                       # both fused kernels, whatever the library would pick
        monkeypatch.setenv("CMN_STEP_KERNEL", mode)
        plan = B.Plan(numel, 2, 2, 256, "f16")
        for t in range(len(numel)):
            p[t].copy_(p0[t]); v[t].copy_(v0[t]); m_fused[t].zero_()
        plan.bind(g, p, v, m_fused)
        plan.allreduce_step(lr, mu, 0.0, write_mean_grad=True)
        torch.cuda.synchronize()
        oracle_windows(mode, m_fused, p, v)
        for t in range(len(numel)):
            for name, a, b in (("mean", m_fused, want_m), ("v", v, want_v), ("p", p, want_p)):
                assert torch.equal(a[t].view(torch.int32), b[t].view(torch.int32)), f"{mode} {name}, tensor {t}"


def test_f16_storage_within_2e3_of_unquantised_fp32():
    """Config 4's value distribution (1 % of elements at 100x) on a smaller list: the mean gradient
    from fp16-stored gradients stays within 2e-3 of the float64 mean b of the un-quantised fp32
    draws, relative to max(|b|, mean_k |g_k|) element by element.  (Rounding to binary16 moves
    each normal element by at most 2^-11 = 4.9e-4 of its magnitude and each subnormal by at most
    2^-25, so the mean moves by at most 4.9e-4 * mean_k |g_k| + 3e-8: the bar has 4x headroom.)"""
    import torch
    from paper_1710_11351_amd import binding as B
    from parity_util import gen_all_grads
    import dataclasses
    c4 = wl.config(4)
    numel = [36864, 64, 64, 147456, 1000, 4096, 589824]
    c = dataclasses.replace(wl.custom_config(numel, K=128, n_chunks=128, grad_dtype="f16", cfg=97,
                                             grad_std=c4.grad_std, outlier_frac=c4.outlier_frac), outlier_scale=c4.outlier_scale)
    g16 = gen_all_grads(c, 0)
    g32 = gen_all_grads(c, 0, unquantised=True)
    d_g = [B.upload_tensors(g) for g in g16]
    d_p = B.upload_tensors(wl.gen_params(c)); d_v = B.upload_tensors(wl.gen_velocity(c))
    d_m = [torch.zeros(n, device="cuda") for n in numel]
    plan = B.Plan(numel, c.K, c.n_chunks, 256, "f16")
    plan.bind(d_g, d_p, d_v, d_m)
    plan.allreduce_step(c.lr, c.mu, c.wd, write_mean_grad=True)
    got = B.download_tensors(d_m)
    for t in range(len(numel)):
        st = np.stack([g[t].astype(np.float64) for g in g32])
        want, mag = st.mean(axis=0), np.abs(st).mean(axis=0)
        assert np.all(np.abs(got[t] - want) <= 2e-3 * np.maximum(np.abs(want), mag)), f"tensor {t}"
        assert np.max(np.abs(got[t] - want)) > 0     # the quantisation is really there


def test_config3_resnet50_k32_adam_full_size():
    run_parity(wl.config(3), steps=2, opt="adam", staged=False)


@pytest.mark.parametrize("K", [4, 8])            # a few and several replicas (either kernel kind is also forced, see conftest.py)
def test_range_steps_replayed_from_a_hip_graph_match_eager(K):
    """A launch-bound sequence of small per-layer-group steps captured once into a HIP graph
    and replayed must give the same bits as eager launches, on every replay (the library
    only enqueues kernels on the caller's stream: nothing else ends up in the graph)."""
    import torch
    from paper_1710_11351_amd import binding as B
    from parity_util import DeviceCase, assert_bit_equal, gen_all_grads
    numel = [4096, 64, 64, 36864, 256, 256, 9408, 1000]
    c = wl.custom_config(numel, K=K, n_chunks=4, cfg=87)
    eager, graphed = DeviceCase(c), DeviceCase(c)
    p0, v0 = wl.gen_params(c), wl.gen_velocity(c)
    for dc in (eager, graphed):
        dc.set_state(p0, v0)
    groups = [(6, 8), (3, 6), (0, 3)]
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    grads = gen_all_grads(c, 0)
    for dc in (eager, graphed):
        for k in range(c.K):
            dc.set_grads(k, grads[k])
    torch.cuda.synchronize()
    state_p = [x.clone() for x in graphed.p]; state_v = [x.clone() for x in graphed.v]
    with torch.cuda.stream(stream):
        graph.capture_begin()
        for t0, t1 in groups:
            graphed.plan.allreduce_step_range(t0, t1, c.lr, c.mu, c.wd, mean_dest=B.CMN_MEAN_TO_MEAN_GRADS,
                                              stream=stream)
        graph.capture_end()
    torch.cuda.synchronize()
    for d, s in zip(graphed.p + graphed.v, state_p + state_v):     # capture must not have run anything
        assert torch.equal(d, s)
    for step in range(3):
        grads = gen_all_grads(c, step)
        for dc in (eager, graphed):
            for k in range(c.K):
                dc.set_grads(k, grads[k])
        for t0, t1 in groups:
            eager.plan.allreduce_step_range(t0, t1, c.lr, c.mu, c.wd, mean_dest=B.CMN_MEAN_TO_MEAN_GRADS)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("p", "v", "m"):
            for t, (a, b) in enumerate(zip(graphed.get(getattr(graphed, name)), eager.get(getattr(eager, name)))):
                assert_bit_equal(a, b, f"replay {step} {name}[{t}]")


def test_very_long_tensor_list_uses_the_global_memory_tables():
    """More tensors than the LDS copy of the offsets and pointer tables can hold (3071): pack and
    unpack search the tables in global memory instead; results must not change."""
    rng = np.random.default_rng(5)
    numel = [int(x) for x in rng.integers(0, 9, 5000)] + [4096, 3]
    c = wl.custom_config(numel, K=3, n_chunks=4, cfg=84)
    run_parity(c, steps=1)
    c16 = wl.custom_config(numel[:4000], K=2, n_chunks=3, grad_dtype="f16", cfg=83)
    run_parity(c16, steps=1)


def test_buffer_arguments_are_validated_on_a_bound_plan():
    import torch
    from paper_1710_11351_amd import binding as B
    from parity_util import DeviceCase
    dc = DeviceCase(wl.custom_config([1000, 24], K=2, n_chunks=2, cfg=82))
    L = dc.plan.L
    packed = torch.zeros(2 * L + 64, device="cuda")
    reduced = torch.zeros(L + 64, device="cuda")
    assert B.cmn_pack(dc.plan.h, None) == B.CMN_ENULL
    assert B.cmn_pack(dc.plan.h, packed.data_ptr() + 4) == B.CMN_EALIGN
    assert B.cmn_ring_reduce(dc.plan.h, packed.data_ptr(), reduced.data_ptr() + 16) == B.CMN_EALIGN
    assert B.cmn_scale_unpack(dc.plan.h, None) == B.CMN_ENULL
    assert B.cmn_scale_unpack(dc.plan.h, reduced.data_ptr() + 128) == B.CMN_EALIGN
    assert B.cmn_pack(dc.plan.h, packed) == B.CMN_OK
    assert B.cmn_ring_reduce(dc.plan.h, packed, reduced) == B.CMN_OK
    assert B.cmn_scale_unpack(dc.plan.h, reduced) == B.CMN_OK
    torch.cuda.synchronize()
    # a plan bound without mean gradients refuses the entry points that need them
    dc2 = DeviceCase(wl.custom_config([1000, 24], K=2, n_chunks=2, cfg=82), with_mean=False)
    assert B.cmn_scale_unpack(dc2.plan.h, reduced) == B.CMN_EUNBOUND
    assert B.cmn_momentum_sgd(dc2.plan.h, .1, .9, 0.) == B.CMN_EUNBOUND
    assert B.cmn_allreduce_step(dc2.plan.h, .1, .9, 0., B.CMN_MEAN_TO_MEAN_GRADS) == B.CMN_EUNBOUND
    assert B.cmn_allreduce_step(dc2.plan.h, .1, .9, 0., B.CMN_MEAN_NONE) == B.CMN_OK
    torch.cuda.synchronize()


def test_a_thousand_replicas():
    c = wl.custom_config([3000, 1, 2100], K=1000, n_chunks=7, cfg=78)
    run_parity(c, steps=1)
