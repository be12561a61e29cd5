"""cmn_allreduce_step_noalloc (the entry point for callers that cannot allocate device memory or bind a
workspace) against cmn_allreduce_step on the same inputs, bit for bit, through the C-ABI.  The file's name
makes pytest collect it last: it shares one array per GPU between all its calls."""
import numpy as np
import pytest

from paper_1710_11351_amd import binding as B
from paper_1710_11351_amd import workloads as wl
from parity_util import DeviceCase, assert_bit_equal, gen_all_grads

pytestmark = pytest.mark.gpu


def _pair(c, misalign=0):
    """Two identical device copies of one workload: `ref` is bound to a workspace the usual way, `na` only
    owns tensors (its plan is created but never bound)."""
    ref, na = DeviceCase(c, misalign=misalign), DeviceCase(c, misalign=misalign)
    na_plan = B.Plan(c.numel, c.K, c.n_chunks, c.align_bytes, c.grad_dtype)
    p0, v0 = wl.gen_params(c), wl.gen_velocity(c)
    for dc in (ref, na):
        dc.set_state(p0, v0)
    return ref, na, na_plan


def _step_both(c, ref, na, na_plan, step, mean_dest):
    grads = gen_all_grads(c, step)
    for dc in (ref, na):
        for k in range(c.K):
            dc.set_grads(k, grads[k])
        for m in dc.m:
            m.fill_(-3.0)
    ref.plan.allreduce_step(c.lr, c.mu, c.wd, mean_dest=mean_dest)
    na_plan.allreduce_step_noalloc(na.grads, na.p, na.v, na.m if mean_dest == B.CMN_MEAN_TO_MEAN_GRADS else None,
                                   c.lr, c.mu, c.wd, mean_dest=mean_dest)
    lists = [("p", ref.p, na.p), ("v", ref.v, na.v), ("mean", ref.m, na.m)]
    if mean_dest == B.CMN_MEAN_TO_ALL_REPLICAS:
        lists += [(f"replica {k}", ref.grads[k], na.grads[k]) for k in range(c.K)]
    for name, a, b in lists:
        for t, (x, y) in enumerate(zip(na.get(b), ref.get(a))):
            assert_bit_equal(x, y, f"{c.name} step {step} {name}[{t}]")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_two_calls_in_a_row_the_second_on_a_smaller_list(dtype):
    """The array keeps the first call's tables; the second call (fewer and shorter tensors, fewer replicas,
    another kernel kind) must overwrite what it needs and give cmn_allreduce_step's bits."""
    import torch
    big = wl.custom_config([300_000, 5, 0, 150_001, 64, 70_000, 7, 2049] * 9, K=9, n_chunks=5, grad_dtype=dtype,
                           cfg=71, wd=1e-3)                              # 4.7 M elements: the persistent two-phase kernel
    small = wl.custom_config([5000, 1, 3, 1025], K=3, n_chunks=2, grad_dtype=dtype, cfg=72)   # one-pass kernel
    rb, nb, pb = _pair(big, misalign=1)
    rs, ns, ps = _pair(small)
    _step_both(big, rb, nb, pb, 0, B.CMN_MEAN_TO_MEAN_GRADS)
    _step_both(small, rs, ns, ps, 0, B.CMN_MEAN_TO_MEAN_GRADS)
    _step_both(small, rs, ns, ps, 1, B.CMN_MEAN_NONE)                  # tables already resident: no rewrite
    _step_both(big, rb, nb, pb, 1, B.CMN_MEAN_TO_ALL_REPLICAS)         # back to the large list
    _step_both(big, rb, nb, pb, 2, B.CMN_MEAN_NONE)
    # same plan, other tensors: the tables are rebuilt for the new addresses
    rb2, nb2, _ = _pair(big)
    _step_both(big, rb2, nb2, pb, 0, B.CMN_MEAN_TO_MEAN_GRADS)
    torch.cuda.synchronize()


def test_back_to_back_calls_without_synchronisation_between_them():
    """Table writes and step kernels of successive calls are ordered by the stream alone."""
    import torch
    a = wl.custom_config([40_000, 333, 4096], K=4, n_chunks=4, cfg=70)
    b = wl.custom_config([1000, 24], K=2, n_chunks=2, cfg=69)
    ra, na, pa = _pair(a)
    rb, nb, pb = _pair(b)
    for dc_pair, c in (((ra, na), a), ((rb, nb), b)):
        g = gen_all_grads(c, 0)
        for dc in dc_pair:
            for k in range(c.K):
                dc.set_grads(k, g[k])
    torch.cuda.synchronize()
    for _ in range(3):                                                  # a, b, a, b, a, b: every call rewrites the tables
        pa.allreduce_step_noalloc(na.grads, na.p, na.v, None, a.lr, a.mu, a.wd)
        pb.allreduce_step_noalloc(nb.grads, nb.p, nb.v, None, b.lr, b.mu, b.wd)
        ra.plan.allreduce_step(a.lr, a.mu, a.wd)
        rb.plan.allreduce_step(b.lr, b.mu, b.wd)
    for ref, got in ((ra, na), (rb, nb)):
        for t, (x, y) in enumerate(zip(got.get(got.p) + got.get(got.v), ref.get(ref.p) + ref.get(ref.v))):
            assert_bit_equal(x, y, f"state {t}")


def test_config3_resnet50_k32_full_size_matches_the_bound_step():
    """The benchmark workload (1.7 MB of tables, 25,052 tiles, two-phase kernel) through the no-allocation entry."""
    c = wl.config(3)
    ref, na, plan = _pair(c)
    _step_both(c, ref, na, plan, 0, B.CMN_MEAN_NONE)
    _step_both(c, ref, na, plan, 1, B.CMN_MEAN_TO_MEAN_GRADS)


def test_captured_into_a_hip_graph_and_replayed_between_eager_calls():
    """Under stream capture the table writes and the step kernels become kernel nodes of the graph; every replay
    rewrites the array for its own plan, and eager calls of another plan in between rewrite it for theirs (after a
    capture the host never assumes it knows what the array holds)."""
    import torch
    a = wl.custom_config([4096, 64, 36864, 256, 9408, 1000], K=4, n_chunks=4, cfg=68)
    b = wl.custom_config([1000, 24, 5000], K=3, n_chunks=2, cfg=67)
    ra, na, pa = _pair(a)
    rb, nb, pb = _pair(b)
    for (ref, got), c in (((ra, na), a), ((rb, nb), b)):
        g = gen_all_grads(c, 0)
        for dc in (ref, got):
            for k in range(c.K):
                dc.set_grads(k, g[k])
    pb.allreduce_step_noalloc(nb.grads, nb.p, nb.v, None, b.lr, b.mu, b.wd)          # the array holds b's tables
    rb.plan.allreduce_step(b.lr, b.mu, b.wd)
    torch.cuda.synchronize()
    stream, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        graph.capture_begin()
        pa.allreduce_step_noalloc(na.grads, na.p, na.v, na.m, a.lr, a.mu, a.wd, mean_dest=B.CMN_MEAN_TO_MEAN_GRADS,
                                  stream=stream)
        graph.capture_end()
    torch.cuda.synchronize()
    for step in range(3):
        g = gen_all_grads(a, step + 1)
        for dc in (ra, na):
            for k in range(a.K):
                dc.set_grads(k, g[k])
        torch.cuda.synchronize()
        graph.replay()
        ra.plan.allreduce_step(a.lr, a.mu, a.wd, mean_dest=B.CMN_MEAN_TO_MEAN_GRADS)
        torch.cuda.synchronize()
        pb.allreduce_step_noalloc(nb.grads, nb.p, nb.v, None, b.lr, b.mu, b.wd)      # eager, other plan, same array
        rb.plan.allreduce_step(b.lr, b.mu, b.wd)
        torch.cuda.synchronize()
        for ref, got, name in ((ra, na, "graph"), (rb, nb, "eager")):
            for t, (x, y) in enumerate(zip(got.get(got.p) + got.get(got.v) + got.get(got.m),
                                           ref.get(ref.p) + ref.get(ref.v) + ref.get(ref.m))):
                assert_bit_equal(x, y, f"replay {step} {name} tensor {t}")


def test_vgg16_list_uses_half_of_the_table_array_full_size():
    """VGG-16's 135 k tiles need 8.7 MB of the 16 MiB array (about 2,400 table-writing launches on the first call)."""
    import dataclasses
    c = dataclasses.replace(wl.config(5), K=2, n_chunks=2, name="vgg16_k2_f32")
    ref, na, plan = _pair(c)
    assert 8_000_000 < plan.workspace_bytes < B.CMN_NOALLOC_SCRATCH_BYTES
    _step_both(c, ref, na, plan, 0, B.CMN_MEAN_NONE)
    _step_both(c, ref, na, plan, 1, B.CMN_MEAN_TO_MEAN_GRADS)
