"""Host-side tests of the C-ABI library: they need no GPU and launch nothing."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_1710_11351_amd import binding as B
from paper_1710_11351_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "cmn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(cmn_[a-z_]+)\s*\(", text)))
    assert {"cmn_pack", "cmn_ring_reduce", "cmn_scale_unpack", "cmn_momentum_sgd", "cmn_allreduce_step",
            "cmn_plan_create", "cmn_plan_bind", "cmn_plan_destroy", "cmn_strerror"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), f"libcmn.so does not export {n}"
        assert hasattr(B, n), f"the Python binding has no function named {n}"


def test_strerror_is_total():
    for s in range(-9, 2):
        assert isinstance(B.cmn_strerror(s), str) and B.cmn_strerror(s)
    assert B.cmn_strerror(B.CMN_OK) == "ok"


@pytest.mark.parametrize("args,status", [
    (dict(numel=[4], K=0, n_chunks=1), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=0), B.CMN_EINVAL),
    (dict(numel=[4, -1], K=1, n_chunks=1), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=1, align_bytes=48), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=1, align_bytes=8), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=1, grad_dtype=7), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=1, grad_dtype=-1), B.CMN_EINVAL),
    (dict(numel=[4], K=1, n_chunks=1, ring_rotate=2), B.CMN_EINVAL),
    (dict(numel=[4], K=5000, n_chunks=1), B.CMN_ESIZE),
    (dict(numel=[1 << 50], K=1, n_chunks=1), B.CMN_ESIZE),
])
def test_plan_create_rejects(args, status):
    rc, h = B.cmn_plan_create(**args)
    assert rc == status and not h.value


def test_null_arguments():
    L = B.lib()
    assert L.cmn_plan_create(None, 0, None, 1, 1, 256, 0, 1) == B.CMN_ENULL
    import ctypes
    h = ctypes.c_void_p()
    assert L.cmn_plan_create(ctypes.byref(h), 2, None, 1, 1, 256, 0, 1) == B.CMN_ENULL
    assert B.cmn_plan_total_elems(None) == -1 and B.cmn_plan_workspace_bytes(None) == 0
    assert B.cmn_plan_destroy(None) == B.CMN_OK
    for call in (lambda: B.cmn_pack(None, 256, 0), lambda: B.cmn_ring_reduce(None, 256, 512, 0),
                 lambda: B.cmn_scale_unpack(None, 256, 0), lambda: B.cmn_momentum_sgd(None, .1, .9, 0., 0),
                 lambda: B.cmn_allreduce_step(None, .1, .9, 0., False, 0)):
        assert call() == B.CMN_ENULL


def test_kernel_entry_points_refuse_an_unbound_plan():
    p = B.Plan([100, 28], 2, 2)
    assert B.cmn_pack(p.h, 256, 0) == B.CMN_EUNBOUND
    assert B.cmn_scale_unpack(p.h, 256, 0) == B.CMN_EUNBOUND
    assert B.cmn_momentum_sgd(p.h, .1, .9, 0., 0) == B.CMN_EUNBOUND
    assert B.cmn_allreduce_step(p.h, .1, .9, 0., False, 0) == B.CMN_EUNBOUND
    # argument checks of the one staged entry point that needs no binding (it works on its two buffers alone) ...
    assert B.cmn_ring_reduce(p.h, None, 512, 0) == B.CMN_ENULL
    assert B.cmn_ring_reduce(p.h, 260, 512, 0) == B.CMN_EALIGN
    # ... except for int8 storage, whose scales come with a binding
    assert B.cmn_ring_reduce(B.Plan([100, 28], 2, 2, 256, "i8s").h, 256, 512, 0) == B.CMN_EUNBOUND
    assert B.cmn_plan_bind(p.h, None, None, None, None, None, 0) == B.CMN_ENULL
    assert B.cmn_plan_bind(p.h, 260, None, None, None, None, 0) == B.CMN_EALIGN
    assert B.cmn_plan_bind(p.h, 256, None, [1024, 2048], None, None, 0) == B.CMN_ENULL   # p without v
    assert B.cmn_plan_bind(p.h, 256, [1024, 0, 4096, 8192], None, None, None, 0) == B.CMN_ENULL
    assert B.cmn_plan_bind(p.h, 256, None, [1024, 2050], [4096, 8192], None, 0) == B.CMN_EALIGN


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


@pytest.mark.parametrize("row", _rows("geometry.txt"), ids=lambda r: "cfg" + r[0])
def test_plan_geometry_matches_hand_worked_table(row):
    c = wl.config(int(row[0]))
    p = B.Plan(c.numel, c.K, c.n_chunks, c.align_bytes, c.grad_dtype)
    assert (p.T, p.N, p.chunk_elems, p.L) == (int(row[2]), int(row[3]), int(row[6]), int(row[7]))
    assert p.workspace_bytes % 256 == 0 and p.workspace_bytes >= 256


def test_plan_geometry_agrees_with_oracle_on_random_lists():
    rng = np.random.default_rng(0)
    for _ in range(50):
        T = int(rng.integers(0, 12))
        numel = [int(x) for x in rng.choice([0, 1, 3, 63, 64, 65, 1000, 4097], T)]
        C = int(rng.integers(1, 9))
        dt = ["f32", "f16", "bf16", "i8s"][int(rng.integers(0, 4))]
        align = int(rng.choice([16, 64, 256, 1024]))
        p = B.Plan(numel, int(rng.integers(1, 9)), C, align, dt)
        g = oracle.Geometry(numel, C, align, dt)
        assert (p.N, p.chunk_elems, p.L) == (g.N, g.chunk_elems, g.L)


def _fake_ptrs(numel, base, elem_bytes, misalign=0):
    out, a = [], base
    for n in numel:
        out.append(a + misalign * elem_bytes if n else 0)
        a += ((n * elem_bytes + 511) // 512 + 1) * 512
    return out, a


@pytest.mark.parametrize("dtype,rot", [("f32", 1), ("f32", 0), ("f16", 1)])
def test_tile_table_covers_every_element_once_inside_one_chunk(dtype, rot):
    numel = [5, 0, 5000, 1, 64, 12345, 7]
    K, C = 3, 5
    p = B.Plan(numel, K, C, 256, dtype, rot)
    eb = 2 if dtype == "f16" else 4
    vec = 16 // eb
    base = 1 << 20
    grads = []
    for k in range(K):
        g, base = _fake_ptrs(numel, base, eb)
        grads += g
    pp, base = _fake_ptrs(numel, base, 4)
    vp, base = _fake_ptrs(numel, base, 4)
    mp, base = _fake_ptrs(numel, base, 4)
    sp, base = _fake_ptrs(numel, base, 4)
    rc, tiles = B.cmn_plan_describe_tiles(p.h, grads, pp, vp, mp, sp)
    assert rc == B.CMN_OK and len(tiles) == p.tile_count
    off = np.concatenate([[0], np.cumsum(numel)])
    covered = {t: 0 for t in range(len(numel))}
    for tl in tiles:
        t, e0, ln = int(tl["tensor"]), int(tl["e0"]), int(tl["len"])
        assert ln > 0 and covered[t] == e0            # in order, no gap, no overlap
        covered[t] = e0 + ln
        c_first, c_last = (off[t] + e0) // p.chunk_elems, (off[t] + e0 + ln - 1) // p.chunk_elems
        assert c_first == c_last
        assert int(tl["start_rank"]) == (c_first % K if rot else 0)
        # all fake bases are 512-byte aligned, so the head only depends on e0
        assert int(tl["head"][B.CMN_HEAD_STEP]) == (-e0) % vec and int(tl["head"][B.CMN_HEAD_STEP_MEAN]) == (-e0) % vec
        assert int(tl["head"][B.CMN_HEAD_ADAM]) == (-e0) % vec and int(tl["head"][B.CMN_HEAD_ADAM_MEAN]) == (-e0) % vec
        assert int(tl["head"][B.CMN_HEAD_SGD]) == (-e0) % 4 and int(tl["head"][B.CMN_HEAD_ADAM_OPT]) == (-e0) % 4
    assert [covered[t] for t in range(len(numel))] == numel


def test_tile_heads_follow_pointer_alignment():
    numel = [1000]
    p = B.Plan(numel, 2, 1)
    a = 1 << 20
    H = lambda tiles, i: int(tiles[0]["head"][i])
    # both replicas, p and v start 3 elements past a 16-byte boundary: one leading element
    rc, tiles = B.cmn_plan_describe_tiles(p.h, [a + 12, 2 * a + 12], [3 * a + 12], [4 * a + 12], [5 * a + 12])
    assert rc == 0 and H(tiles, B.CMN_HEAD_STEP) == 1 and H(tiles, B.CMN_HEAD_SGD) == 1
    assert H(tiles, B.CMN_HEAD_ADAM) == -1                       # no second moments given
    # replicas disagree: no common alignment
    rc, tiles = B.cmn_plan_describe_tiles(p.h, [a + 12, 2 * a + 8], [3 * a + 12], [4 * a + 12], [5 * a + 12])
    assert rc == 0 and H(tiles, B.CMN_HEAD_STEP) == -1 and H(tiles, B.CMN_HEAD_SGD) == 1
    # mean gradient misaligned differently: only the variants that touch it lose the vector path
    rc, tiles = B.cmn_plan_describe_tiles(p.h, [a, 2 * a], [3 * a], [4 * a], [5 * a + 4], [6 * a])
    assert rc == 0 and H(tiles, B.CMN_HEAD_STEP) == 0 and H(tiles, B.CMN_HEAD_ADAM) == 0
    assert H(tiles, B.CMN_HEAD_STEP_MEAN) == -1 and H(tiles, B.CMN_HEAD_SGD) == -1
    assert H(tiles, B.CMN_HEAD_ADAM_MEAN) == -1 and H(tiles, B.CMN_HEAD_ADAM_OPT) == -1
    # second moments misaligned: only Adam variants lose it
    rc, tiles = B.cmn_plan_describe_tiles(p.h, [a, 2 * a], [3 * a], [4 * a], [5 * a], [6 * a + 8])
    assert rc == 0 and H(tiles, B.CMN_HEAD_STEP_MEAN) == 0 and H(tiles, B.CMN_HEAD_ADAM) == -1
    # unbound arrays
    rc, tiles = B.cmn_plan_describe_tiles(p.h, None, None, None, None)
    assert rc == 0 and H(tiles, B.CMN_HEAD_STEP) == -1
    rc, _ = B.cmn_plan_describe_tiles(p.h, [a + 2, 2 * a], None, None, None)
    assert rc == B.CMN_EALIGN


def test_range_and_adam_argument_checks():
    p = B.Plan([100, 28, 7], 2, 2)
    assert B.cmn_allreduce_step_range(None, 0, 1, .1, .9, 0., 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_step_range(p.h, 0, 1, .1, .9, 0., 0, 0) == B.CMN_EUNBOUND
    assert B.cmn_allreduce_adam_step(p.h, 1e-3, .9, .999, 1e-8, 0., 0, 0, 0) == B.CMN_EINVAL      # t < 1
    assert B.cmn_allreduce_adam_step(None, 1e-3, .9, .999, 1e-8, 0., 1, 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_adam_step(p.h, 1e-3, .9, .999, 1e-8, 0., 1, 0, 0) == B.CMN_EUNBOUND
    assert B.cmn_adam(p.h, 1e-3, .9, .999, 1e-8, 0., 1, 0) == B.CMN_EUNBOUND
    assert B.cmn_adam(p.h, 1e-3, .9, .999, 1e-8, 0., 0, 0) == B.CMN_EINVAL
    assert B.cmn_plan_bind_adam(p.h, [1024, 2048, 4096], 0) == B.CMN_EUNBOUND                    # before cmn_plan_bind
    assert B.cmn_plan_bind_adam(p.h, None, 0) == B.CMN_ENULL


def test_kernel_kind_follows_the_measured_rule(monkeypatch):
    """Two-phase fused kernel from about 44 gradient bytes per element while parameters and state
    stay within twice the memory-side cache, from 32 bytes beyond that, never for int8; the environment can force
    either kind where it applies."""
    from paper_1710_11351_amd import workloads as wl
    monkeypatch.delenv("CMN_STEP_KERNEL", raising=False)
    small, big = wl.config(3).numel, wl.config(5).numel
    kind = lambda numel, K, dt="f32": B.Plan(numel, K, K, 256, dt).step_kernel_kind
    assert [kind(small, K) for K in (1, 4, 5, 8, 10, 11, 32)] == [3, 3, 1, 1, 1, 2, 2]    # 3: one pass, state requested first
    assert [kind(small, K, "f16") for K in (16, 21, 22, 128)] == [1, 1, 2, 2]
    assert [kind(big, K) for K in (4, 7, 8, 16)] == [1, 1, 2, 2]
    assert [kind(big, K, "bf16") for K in (8, 15, 16)] == [1, 1, 2]
    adam = lambda numel, K, dt="f32": B.Plan(numel, K, K, 256, dt).adam_step_kernel_kind
    assert [adam(small, K) for K in (4, 8, 10, 11, 32)] == [3, 1, 1, 2, 2]     # both moments: 306 MB, still served by the cache
    def to_all(K):
        p = B.Plan(small, K, K)
        return B.cmn_plan_step_kernel_kind(p.h, 0, B.CMN_MEAN_TO_ALL_REPLICAS)
    assert [to_all(K) for K in (7, 8)] == [1, 2]                       # heavy stores: like state beyond the cache
    assert kind(small, 128, "i8s") == 1 and kind(small, 4, "i8s") == 1 and kind(small, 4, "f16") == 1
    assert B.cmn_plan_step_kernel_kind(B.Plan(small, 4, 4).h, 0, B.CMN_MEAN_TO_ALL_REPLICAS) == 1
    assert B.cmn_plan_step_kernel_kind(B.Plan(small, 4, 4).h, 0, B.CMN_MEAN_TO_MEAN_GRADS) == 3
    assert B.cmn_plan_step_kernel_kind(None) == -1
    # a launch over few tiles takes the one-pass kernel whatever the plan-wide rule says, and the
    # query reports it: whole small lists, and small layer groups of a large list
    assert B.Plan([4095 * 1024], 32, 1).step_kernel_kind == 1 and B.Plan([4096 * 1024], 32, 1).step_kernel_kind == 2
    p = B.Plan(small, 32, 32)
    assert B.cmn_plan_range_kernel_kind(p.h, 0, len(small), 0, 0) == 2
    assert B.cmn_plan_range_kernel_kind(p.h, 0, 10, 0, 0) == 1           # the stem and first bottleneck: 75 k elements
    assert B.cmn_plan_range_kernel_kind(p.h, 5, 5, 0, 0) == 1
    assert B.cmn_plan_range_kernel_kind(p.h, 3, 2, 0, 0) == -1 and B.cmn_plan_range_kernel_kind(p.h, 0, 162, 0, 0) == -1
    # launches per fused step: one per round of the persistent grid (512 workgroups x 50 tiles when the device
    # cannot be asked, as here), one for the one-pass kernel, none for an empty range
    assert B.cmn_plan_range_launch_count(p.h, 0, len(small), 0, 0) == 1 and B.cmn_plan_range_launch_count(p.h, 0, 10, 0, 0) == 1
    assert B.cmn_plan_range_launch_count(p.h, 5, 5, 0, 0) == 0 and B.cmn_plan_range_launch_count(p.h, 0, 162, 0, 0) == -1
    pv = B.Plan(big, 16, 16)
    assert B.cmn_plan_range_launch_count(pv.h, 0, len(big), 0, 0) == 6 and B.cmn_plan_range_launch_count(pv.h, 0, len(big), 1, 0) == 6
    assert B.cmn_plan_range_launch_count(B.Plan(small, 128, 128, 256, "f16").h, 0, len(small), 0, 0) == 1
    monkeypatch.setenv("CMN_STEP_KERNEL", "two_phase")
    assert kind(small, 2) == 2 and kind(small, 128, "i8s") == 1 and kind([100], 2) == 2
    monkeypatch.setenv("CMN_STEP_KERNEL", "stream")
    assert kind(small, 32) == 1 and kind(big, 16) == 1


def test_noalloc_step_checks_its_arguments_before_touching_the_gpu():
    """The entry point for callers that cannot allocate keeps its tables in a 16 MiB array inside the
    library: plans whose tables are larger are refused, and so are int8 plans and missing lists."""
    numel = [1000, 24]
    p = B.Plan(numel, 2, 2)
    g, pp, vp = [1024, 8192, 16384, 32768], [65536, 131072], [262144, 524288]
    assert B.cmn_allreduce_step_noalloc(None, g, pp, vp, None, .1, .9, 0., 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_step_noalloc(p.h, None, pp, vp, None, .1, .9, 0., 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_step_noalloc(p.h, g, None, vp, None, .1, .9, 0., 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_step_noalloc(p.h, g, pp, [262144, 0], None, .1, .9, 0., 0, 0) == B.CMN_ENULL
    assert B.cmn_allreduce_step_noalloc(p.h, g, [65538, 131072], vp, None, .1, .9, 0., 0, 0) == B.CMN_EALIGN
    assert B.cmn_allreduce_step_noalloc(p.h, g, pp, vp, None, .1, .9, 0., 3, 0) == B.CMN_EINVAL
    assert B.cmn_allreduce_step_noalloc(p.h, g, pp, vp, None, .1, .9, 0., B.CMN_MEAN_TO_MEAN_GRADS, 0) == B.CMN_EUNBOUND
    p8 = B.Plan(numel, 2, 2, 256, "i8s")
    assert B.cmn_allreduce_step_noalloc(p8.h, g, pp, vp, None, .1, .9, 0., 0, 0) == B.CMN_EINVAL
    # one tile record of 64 bytes per 1024 fp32 elements: 300 M elements need more than 16 MiB of tables
    big = B.Plan([300_000_000], 2, 2)
    assert big.workspace_bytes > B.CMN_NOALLOC_SCRATCH_BYTES
    assert B.cmn_allreduce_step_noalloc(big.h, [1024, 2048], [4096], [8192], None, .1, .9, 0., 0, 0) == B.CMN_ESIZE
    from paper_1710_11351_amd import workloads as wl
    for cfg in (3, 4, 5):                            # the benchmark workloads all fit
        c = wl.config(cfg)
        assert B.Plan(c.numel, c.K, c.n_chunks, 256, c.grad_dtype).workspace_bytes <= B.CMN_NOALLOC_SCRATCH_BYTES
    empty = B.Plan([0, 0], 2, 2)                     # nothing to do: no GPU call is made
    assert B.cmn_allreduce_step_noalloc(empty.h, [0, 0, 0, 0], [0, 0], [0, 0], None, .1, .9, 0., 0, 0) == B.CMN_OK


def test_empty_plans():
    for numel in ([], [0, 0]):
        p = B.Plan(numel, 4, 4)
        assert (p.N, p.L, p.chunk_elems, p.tile_count) == (0, 0, 0, 0)
        assert p.workspace_bytes >= 256


def test_plain_c_client_links_and_runs(tmp_path):
    """include/cmn.h compiles as C11 and a C program can drive the library with no C++/Python."""
    import subprocess
    exe = tmp_path / "abi_check"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_check.c"), "-o", str(exe), "-L", libdir, "-lcmn",
                    f"-Wl,-rpath,{libdir}"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and "abi_check ok" in r.stdout, r.stdout + r.stderr


# ------------------------------------------------------------------ property test of the tile table
from hypothesis import given, settings, strategies as st


@settings(max_examples=120, deadline=None)
@given(numel=st.lists(st.sampled_from([0, 1, 3, 7, 64, 100, 1023, 1024, 1025, 4097, 20000]), min_size=1, max_size=9),
       K=st.integers(1, 9), C=st.integers(1, 7), dtype=st.sampled_from(["f32", "f16", "bf16", "i8s"]),
       rot=st.integers(0, 1), mis=st.lists(st.integers(0, 7), min_size=4, max_size=4))
def test_tile_table_invariants_hold_for_any_list(numel, K, C, dtype, rot, mis):
    """Coverage, chunk confinement, fold start and vector alignment of every tile, for arbitrary
    lists, replica counts, chunk counts, storage types and base misalignments."""
    eb = {"f32": 4, "f16": 2, "bf16": 2, "i8s": 1}[dtype]
    vec = 16 // eb
    p = B.Plan(numel, K, C, 256, dtype, rot)
    base = 1 << 24
    grads = []
    for k in range(K):
        g, base = _fake_ptrs(numel, base, eb, misalign=mis[0] if k % 2 == 0 else mis[1])
        grads.append(g)
    pp, base = _fake_ptrs(numel, base, 4, misalign=mis[2])
    vp, base = _fake_ptrs(numel, base, 4, misalign=mis[2])
    mp, base = _fake_ptrs(numel, base, 4, misalign=mis[3])
    sp, base = _fake_ptrs(numel, base, 4, misalign=mis[2])
    rc, tiles = B.cmn_plan_describe_tiles(p.h, [a for g in grads for a in g], pp, vp, mp, sp)
    assert rc == B.CMN_OK and len(tiles) == p.tile_count
    off = np.concatenate([[0], np.cumsum(numel)])
    covered = [0] * len(numel)
    streams = {B.CMN_HEAD_STEP: lambda t: [(g[t], eb) for g in grads] + [(pp[t], 4), (vp[t], 4)],
               B.CMN_HEAD_STEP_MEAN: lambda t: [(g[t], eb) for g in grads] + [(pp[t], 4), (vp[t], 4), (mp[t], 4)],
               B.CMN_HEAD_SGD: lambda t: [(mp[t], 4), (pp[t], 4), (vp[t], 4)],
               B.CMN_HEAD_ADAM: lambda t: [(g[t], eb) for g in grads] + [(pp[t], 4), (vp[t], 4), (sp[t], 4)],
               B.CMN_HEAD_ADAM_MEAN: lambda t: [(g[t], eb) for g in grads] + [(pp[t], 4), (vp[t], 4), (sp[t], 4), (mp[t], 4)],
               B.CMN_HEAD_ADAM_OPT: lambda t: [(mp[t], 4), (pp[t], 4), (vp[t], 4), (sp[t], 4)]}
    for tl in tiles:
        t, e0, ln, c = int(tl["tensor"]), int(tl["e0"]), int(tl["len"]), int(tl["chunk"])
        assert 0 < ln <= 256 * vec and covered[t] == e0
        covered[t] += ln
        assert (off[t] + e0) // p.chunk_elems == c == (off[t] + e0 + ln - 1) // p.chunk_elems and c < C
        assert int(tl["start_rank"]) == (c % K if rot else 0)
        for variant, lst in streams.items():
            h = int(tl["head"][variant])
            w = 4 if variant in (B.CMN_HEAD_SGD, B.CMN_HEAD_ADAM_OPT) else vec
            assert -1 <= h < w
            if h >= 0:   # element e0 + h starts a 16-byte vector on every stream of the variant
                for addr, es in lst(t):
                    assert (addr + (e0 + h) * es) % 16 == 0
            else:        # no head makes all streams 16-byte aligned at once
                assert not any(all((addr + (e0 + hh) * es) % 16 == 0 for addr, es in lst(t)) for hh in range(w))
    assert covered == list(numel)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: asking for more exits with a message, before any GPU work."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def _bench_module():
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    return bench


def test_bench_quotes_counter_traffic_only_for_the_profiled_workload_and_kernel(tmp_path):
    """roofline.traffic comes from a committed rocprofv3 counter summary and is null unless the workload and
    the kernel instance that was launched are the ones that summary measured."""
    bench = _bench_module()
    (tmp_path / "some_pmc.txt").write_text(
        "prose ...\nTRAFFIC workload=resnet50_k32_f32 kernel=k_step_two_phase<0,8,0,0> launches_per_step=1 bytes_per_step=3691800000\n"
        "TRAFFIC workload=vgg16_k16_f32 kernel=k_step_two_phase<0,8,0,0> launches_per_step=6 bytes_per_step=11100000000\n")
    (tmp_path / "kernel_stats.txt").write_text("TRAFFIC workload=resnet50_k32_f32 kernel=k_step<0,16,0,0,0> launches_per_step=1 bytes_per_step=1\n")
    d = str(tmp_path)
    got, src = bench.profiled_traffic("resnet50_k32_f32", "k_step_two_phase<0,8,0,0>", 1, d)
    assert got == 3_691_800_000 and src.endswith("some_pmc.txt")
    assert bench.profiled_traffic("vgg16_k16_f32", "k_step_two_phase<0,8,0,0>", 6, d)[0] == 11_100_000_000
    assert bench.profiled_traffic("resnet50_k32_f32", "k_step<0,16,0,0,0>", 1, d) == (None, None)      # forced one-pass kernel
    assert bench.profiled_traffic("resnet50_k32_f32+bf16", "k_step_two_phase<2,8,0,0>", 1, d) == (None, None)   # other storage type
    assert bench.profiled_traffic("resnet50_k32_f32", "k_step_two_phase<0,8,1,0>", 1, d) == (None, None)  # mean gradient stored
    assert bench.profiled_traffic("vgg16_k16_f32", "k_step_two_phase<0,8,0,0>", 5, d) == (None, None)     # another launch split
    assert bench.step_kernel_name("f32", 2, 0, "sgd") == "k_step_two_phase<0,8,0,0>"
    assert bench.step_kernel_name("i8s", 1, 1, "adam") == "k_step<3,16,0,1,1>"
    # every summary under profiles/ that carries such lines parses, and names a kernel of this library
    import glob
    for path in glob.glob(os.path.join(ROOT, "profiles", "*pmc*.txt")):
        for line in open(path):
            if line.startswith("TRAFFIC "):
                kv = dict(x.split("=", 1) for x in line.split()[1:])
                assert kv["kernel"].startswith("k_step") and int(kv["bytes_per_step"]) > 0 and int(kv["launches_per_step"]) > 0


def test_algorithmic_bytes_match_the_stated_formulas():
    """bench.py prices a launch at (K*e_g + 16)*N bytes (+4N with the mean stored, +K*e_g*N handed back to all
    replicas, +8N for Adam's second moment) and the staged entry points at 2*K*e_g*N, (K*e_g+4)*N, 8N, 20N."""
    from paper_1710_11351_amd import workloads as wl
    bench = _bench_module()
    c = wl.config(3)
    N, K = c.N, c.K
    assert bench.algorithmic_bytes(c, "step", 0, "sgd") == (4 * K + 16) * N == 3_680_212_608
    assert bench.algorithmic_bytes(c, "step", 1, "sgd") == (4 * K + 20) * N
    assert bench.algorithmic_bytes(c, "step", 2, "sgd") == (8 * K + 16) * N
    assert bench.algorithmic_bytes(c, "step", 0, "adam") == (4 * K + 24) * N
    assert bench.algorithmic_bytes(c, "pack") == 2 * K * 4 * N
    assert bench.algorithmic_bytes(c, "ring_reduce") == (4 * K + 4) * N
    assert bench.algorithmic_bytes(c, "scale_unpack") == 8 * N
    assert bench.algorithmic_bytes(c, "momentum_sgd") == 20 * N
    c4 = wl.config(4)
    assert bench.algorithmic_bytes(c4, "step", 0, "sgd") == (2 * 128 + 16) * c4.N
