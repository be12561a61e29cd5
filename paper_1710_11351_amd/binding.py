"""ctypes binding of libcmn.so: argument marshalling only.

Module-level functions carry the names of the C entry points declared in
``include/cmn.h``; ``Plan`` bundles a plan handle with the device workspace and
the tensors it was bound to (so they stay alive).  PyTorch is used for device
memory and stream handles, nothing else: every step runs in the HIP kernels.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcmn.so")

CMN_OK, CMN_EINVAL, CMN_ENULL, CMN_ESIZE, CMN_EALIGN, CMN_EUNBOUND, CMN_EHIP, CMN_ENOMEM = 0, -1, -2, -3, -4, -5, -6, -7
CMN_F32, CMN_F16, CMN_BF16, CMN_I8S = 0, 1, 2, 3
_DT = {"f32": CMN_F32, "f16": CMN_F16, "bf16": CMN_BF16, "i8s": CMN_I8S,
       CMN_F32: CMN_F32, CMN_F16: CMN_F16, CMN_BF16: CMN_BF16, CMN_I8S: CMN_I8S}


CMN_MEAN_NONE, CMN_MEAN_TO_MEAN_GRADS, CMN_MEAN_TO_ALL_REPLICAS = 0, 1, 2
(CMN_HEAD_STEP, CMN_HEAD_STEP_MEAN, CMN_HEAD_SGD, CMN_HEAD_ADAM, CMN_HEAD_ADAM_MEAN,
 CMN_HEAD_ADAM_OPT) = range(6)


class cmn_tile(ctypes.Structure):
    _fields_ = [("e0", ctypes.c_int64), ("len", ctypes.c_int32), ("tensor", ctypes.c_int32),
                ("start_rank", ctypes.c_int32), ("chunk", ctypes.c_int32), ("head", ctypes.c_int8 * 8)]


TILE_DTYPE = np.dtype([("e0", "<i8"), ("len", "<i4"), ("tensor", "<i4"), ("start_rank", "<i4"),
                       ("chunk", "<i4"), ("head", "i1", (8,))])


class CmnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {cmn_strerror(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libcmn.so (built in-tree by ``paper_1710_11351_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU or PyTorch fallback for the HIP path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64p, vpp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_void_p)
    L.cmn_plan_create.restype = ctypes.c_int
    L.cmn_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64p, ctypes.c_int, ctypes.c_int,
                                  ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.cmn_plan_destroy.restype = ctypes.c_int
    L.cmn_plan_destroy.argtypes = [vp]
    for name in ("cmn_plan_total_elems", "cmn_plan_padded_elems", "cmn_plan_chunk_elems", "cmn_plan_tile_count"):
        getattr(L, name).restype = ctypes.c_int64
        getattr(L, name).argtypes = [vp]
    L.cmn_plan_step_kernel_kind.restype = ctypes.c_int
    L.cmn_plan_step_kernel_kind.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    L.cmn_plan_range_kernel_kind.restype = ctypes.c_int
    L.cmn_plan_range_kernel_kind.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.cmn_plan_range_launch_count.restype = ctypes.c_int
    L.cmn_plan_range_launch_count.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.cmn_plan_workspace_bytes.restype = ctypes.c_size_t
    L.cmn_plan_workspace_bytes.argtypes = [vp]
    L.cmn_plan_describe_tiles.restype = ctypes.c_int
    L.cmn_plan_describe_tiles.argtypes = [vp, vpp, vpp, vpp, vpp, vpp, ctypes.POINTER(cmn_tile)]
    L.cmn_plan_bind_scales.restype = ctypes.c_int
    L.cmn_plan_bind_scales.argtypes = [vp, vpp, vp]
    L.cmn_plan_bind_adam.restype = ctypes.c_int
    L.cmn_plan_bind_adam.argtypes = [vp, vpp, vp]
    L.cmn_plan_bind.restype = ctypes.c_int
    L.cmn_plan_bind.argtypes = [vp, vp, vpp, vpp, vpp, vpp, vp]
    L.cmn_pack.restype = ctypes.c_int
    L.cmn_pack.argtypes = [vp, vp, vp]
    L.cmn_ring_reduce.restype = ctypes.c_int
    L.cmn_ring_reduce.argtypes = [vp, vp, vp, vp]
    L.cmn_scale_unpack.restype = ctypes.c_int
    L.cmn_scale_unpack.argtypes = [vp, vp, vp]
    L.cmn_momentum_sgd.restype = ctypes.c_int
    L.cmn_momentum_sgd.argtypes = [vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp]
    L.cmn_allreduce_step.restype = ctypes.c_int
    L.cmn_allreduce_step.argtypes = [vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int, vp]
    f = ctypes.c_float
    L.cmn_allreduce_step_range.restype = ctypes.c_int
    L.cmn_allreduce_step_range.argtypes = [vp, ctypes.c_int, ctypes.c_int, f, f, f, ctypes.c_int, vp]
    L.cmn_allreduce_adam_step.restype = ctypes.c_int
    L.cmn_allreduce_adam_step.argtypes = [vp, f, f, f, f, f, ctypes.c_int, ctypes.c_int, vp]
    L.cmn_allreduce_adam_step_range.restype = ctypes.c_int
    L.cmn_allreduce_adam_step_range.argtypes = [vp, ctypes.c_int, ctypes.c_int, f, f, f, f, f, ctypes.c_int,
                                                ctypes.c_int, vp]
    L.cmn_adam.restype = ctypes.c_int
    L.cmn_adam.argtypes = [vp, f, f, f, f, f, ctypes.c_int, vp]
    L.cmn_allreduce_step_noalloc.restype = ctypes.c_int
    L.cmn_allreduce_step_noalloc.argtypes = [vp, vpp, vpp, vpp, vpp, f, f, f, ctypes.c_int, vp]
    L.cmn_strerror.restype = ctypes.c_char_p
    L.cmn_strerror.argtypes = [ctypes.c_int]
    _lib = L
    return L


# ------------------------------------------------------------------ marshalling helpers
def _addr(x) -> Optional[int]:
    """Device/host address of a tensor-like, or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(ptrs: Optional[Sequence]):
    """Host array of addresses for the C side; an array made by an earlier call is passed through, so that a
    caller in a loop can marshal its tensor lists once."""
    if ptrs is None or isinstance(ptrs, ctypes.Array):
        return ptrs
    arr = (ctypes.c_void_p * max(1, len(ptrs)))()
    for i, p in enumerate(ptrs):
        arr[i] = _addr(p)
    return arr


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream)


def ptr_array(ptrs: Sequence):
    """Public form of the marshalling step: tensors / addresses -> a reusable host pointer array."""
    return _ptr_array(ptrs)


# ------------------------------------------------------------------ C entry points, same names
def cmn_strerror(status: int) -> str:
    return lib().cmn_strerror(int(status)).decode()


def cmn_plan_create(numel: Sequence[int], K: int, n_chunks: int, align_bytes: int = 256, grad_dtype=CMN_F32,
                    ring_rotate: int = 1):
    """Returns (status, handle)."""
    arr = np.ascontiguousarray(numel, dtype=np.int64)
    h = ctypes.c_void_p()
    rc = lib().cmn_plan_create(ctypes.byref(h), len(arr), arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               int(K), int(n_chunks), int(align_bytes), int(_DT.get(grad_dtype, grad_dtype)),
                               int(ring_rotate))
    return rc, h


def cmn_plan_destroy(h) -> int:
    return lib().cmn_plan_destroy(h)


def cmn_plan_total_elems(h) -> int:
    return lib().cmn_plan_total_elems(h)


def cmn_plan_padded_elems(h) -> int:
    return lib().cmn_plan_padded_elems(h)


def cmn_plan_chunk_elems(h) -> int:
    return lib().cmn_plan_chunk_elems(h)


def cmn_plan_tile_count(h) -> int:
    return lib().cmn_plan_tile_count(h)


def cmn_plan_step_kernel_kind(h, adam: int = 0, mean_dest: int = 0) -> int:
    return lib().cmn_plan_step_kernel_kind(h, int(adam), int(mean_dest))


def cmn_plan_range_kernel_kind(h, tensor_begin: int, tensor_end: int, adam: int = 0, mean_dest: int = 0) -> int:
    return lib().cmn_plan_range_kernel_kind(h, int(tensor_begin), int(tensor_end), int(adam), int(mean_dest))


def cmn_plan_range_launch_count(h, tensor_begin: int, tensor_end: int, adam: int = 0, mean_dest: int = 0) -> int:
    return lib().cmn_plan_range_launch_count(h, int(tensor_begin), int(tensor_end), int(adam), int(mean_dest))


def cmn_plan_workspace_bytes(h) -> int:
    return lib().cmn_plan_workspace_bytes(h)


def cmn_plan_describe_tiles(h, grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, second_moment_ptrs=None):
    """Returns (status, numpy structured array of tiles).  Pointers are ints or tensors."""
    n = max(0, cmn_plan_tile_count(h))
    out = np.zeros(n, dtype=TILE_DTYPE)
    rc = lib().cmn_plan_describe_tiles(h, _ptr_array(grad_ptrs), _ptr_array(param_ptrs), _ptr_array(vel_ptrs),
                                       _ptr_array(mean_grad_ptrs), _ptr_array(second_moment_ptrs),
                                       out.ctypes.data_as(ctypes.POINTER(cmn_tile)) if n else None)
    return rc, out


def cmn_plan_bind_scales(h, scale_ptrs, stream=None) -> int:
    return lib().cmn_plan_bind_scales(h, _ptr_array(scale_ptrs), _stream(stream))


def cmn_plan_bind_adam(h, second_moment_ptrs, stream=None) -> int:
    return lib().cmn_plan_bind_adam(h, _ptr_array(second_moment_ptrs), _stream(stream))


def cmn_plan_bind(h, dev_workspace, grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, stream=None) -> int:
    return lib().cmn_plan_bind(h, _addr(dev_workspace), _ptr_array(grad_ptrs), _ptr_array(param_ptrs),
                               _ptr_array(vel_ptrs), _ptr_array(mean_grad_ptrs), _stream(stream))


def cmn_pack(h, packed, stream=None) -> int:
    return lib().cmn_pack(h, _addr(packed), _stream(stream))


def cmn_ring_reduce(h, packed, reduced, stream=None) -> int:
    return lib().cmn_ring_reduce(h, _addr(packed), _addr(reduced), _stream(stream))


def cmn_scale_unpack(h, reduced, stream=None) -> int:
    return lib().cmn_scale_unpack(h, _addr(reduced), _stream(stream))


def cmn_momentum_sgd(h, lr: float, mu: float, wd: float, stream=None) -> int:
    return lib().cmn_momentum_sgd(h, lr, mu, wd, _stream(stream))


def cmn_allreduce_step(h, lr: float, mu: float, wd: float, mean_dest: int = CMN_MEAN_NONE, stream=None) -> int:
    return lib().cmn_allreduce_step(h, lr, mu, wd, int(mean_dest), _stream(stream))


def cmn_allreduce_step_range(h, tensor_begin: int, tensor_end: int, lr: float, mu: float, wd: float,
                             mean_dest: int = CMN_MEAN_NONE, stream=None) -> int:
    return lib().cmn_allreduce_step_range(h, int(tensor_begin), int(tensor_end), lr, mu, wd, int(mean_dest),
                                          _stream(stream))


CMN_NOALLOC_SCRATCH_BYTES = 16 * 1024 * 1024


def cmn_allreduce_step_noalloc(h, grad_ptrs, param_ptrs, vel_ptrs, mean_grad_ptrs, lr: float, mu: float, wd: float,
                               mean_dest: int = CMN_MEAN_NONE, stream=None) -> int:
    return lib().cmn_allreduce_step_noalloc(h, _ptr_array(grad_ptrs), _ptr_array(param_ptrs), _ptr_array(vel_ptrs),
                                            _ptr_array(mean_grad_ptrs), lr, mu, wd, int(mean_dest), _stream(stream))


def cmn_allreduce_adam_step(h, alpha, beta1, beta2, eps, wd, t: int, mean_dest: int = CMN_MEAN_NONE,
                            stream=None) -> int:
    return lib().cmn_allreduce_adam_step(h, alpha, beta1, beta2, eps, wd, int(t), int(mean_dest), _stream(stream))


def cmn_allreduce_adam_step_range(h, tensor_begin: int, tensor_end: int, alpha, beta1, beta2, eps, wd, t: int,
                                  mean_dest: int = CMN_MEAN_NONE, stream=None) -> int:
    return lib().cmn_allreduce_adam_step_range(h, int(tensor_begin), int(tensor_end), alpha, beta1, beta2, eps, wd,
                                               int(t), int(mean_dest), _stream(stream))


def cmn_adam(h, alpha, beta1, beta2, eps, wd, t: int, stream=None) -> int:
    return lib().cmn_adam(h, alpha, beta1, beta2, eps, wd, int(t), _stream(stream))


# ------------------------------------------------------------------ convenience wrapper
def _check(rc: int, where: str) -> None:
    if rc != CMN_OK:
        raise CmnError(rc, where)


class Plan:
    """A plan handle plus the device workspace and bound tensors it refers to."""

    def __init__(self, numel: Sequence[int], K: int, n_chunks: int, align_bytes: int = 256, grad_dtype="f32",
                 ring_rotate: int = 1):
        rc, self.h = cmn_plan_create(numel, K, n_chunks, align_bytes, grad_dtype, ring_rotate)
        _check(rc, "cmn_plan_create")
        self.numel = [int(n) for n in numel]
        self.T, self.K, self.C = len(self.numel), int(K), int(n_chunks)
        self.grad_dtype = _DT[grad_dtype]
        self.N = cmn_plan_total_elems(self.h)
        self.L = cmn_plan_padded_elems(self.h)
        self.chunk_elems = cmn_plan_chunk_elems(self.h)
        self.tile_count = cmn_plan_tile_count(self.h)
        self.workspace_bytes = cmn_plan_workspace_bytes(self.h)
        self.step_kernel_kind = cmn_plan_step_kernel_kind(self.h, 0, 0)      # MomentumSGD, average not stored
        self.adam_step_kernel_kind = cmn_plan_step_kernel_kind(self.h, 1, 0)
        self._keep = None

    def close(self) -> None:
        if getattr(self, "h", None) is not None and _lib is not None:
            _lib.cmn_plan_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:   # interpreter shutdown: globals may already be gone
            pass

    def bind(self, grads=None, params=None, vels=None, mean_grads=None, stream=None) -> None:
        """grads[k][t], params[t], vels[t], mean_grads[t]: CUDA tensors (any may be None)."""
        import torch
        ws = torch.empty(self.workspace_bytes, dtype=torch.uint8, device="cuda")
        flat = None if grads is None else [g for row in grads for g in row]
        if grads is not None:
            assert len(grads) == self.K and all(len(r) == self.T for r in grads)
        _check(cmn_plan_bind(self.h, ws, flat, params, vels, mean_grads, stream), "cmn_plan_bind")
        self._keep = (ws, grads, params, vels, mean_grads)

    def pack(self, packed, stream=None) -> None:
        _check(cmn_pack(self.h, packed, stream), "cmn_pack")

    def ring_reduce(self, packed, reduced, stream=None) -> None:
        _check(cmn_ring_reduce(self.h, packed, reduced, stream), "cmn_ring_reduce")

    def scale_unpack(self, reduced, stream=None) -> None:
        _check(cmn_scale_unpack(self.h, reduced, stream), "cmn_scale_unpack")

    def momentum_sgd(self, lr, mu, wd, stream=None) -> None:
        _check(cmn_momentum_sgd(self.h, lr, mu, wd, stream), "cmn_momentum_sgd")

    def allreduce_step(self, lr, mu, wd, write_mean_grad=False, stream=None, mean_dest=None) -> None:
        dest = int(bool(write_mean_grad)) if mean_dest is None else int(mean_dest)
        _check(cmn_allreduce_step(self.h, lr, mu, wd, dest, stream), "cmn_allreduce_step")

    def allreduce_step_range(self, tensor_begin, tensor_end, lr, mu, wd, mean_dest=CMN_MEAN_NONE, stream=None) -> None:
        _check(cmn_allreduce_step_range(self.h, tensor_begin, tensor_end, lr, mu, wd, mean_dest, stream),
               "cmn_allreduce_step_range")

    def allreduce_step_noalloc(self, grads, params, vels, mean_grads, lr, mu, wd, mean_dest=CMN_MEAN_NONE,
                               stream=None) -> None:
        """The fused step on an unbound plan with the library's own table array (see cmn.h)."""
        flat = [g for row in grads for g in row]
        _check(cmn_allreduce_step_noalloc(self.h, flat, params, vels, mean_grads, lr, mu, wd, mean_dest, stream),
               "cmn_allreduce_step_noalloc")

    def bind_scales(self, scales, stream=None) -> None:
        """scales[k]: CUDA float32 tensor of n_chunks scales of replica k (int8 gradient storage)."""
        _check(cmn_plan_bind_scales(self.h, scales, stream), "cmn_plan_bind_scales")
        self._keep = (self._keep, scales)

    def bind_adam(self, second_moments, stream=None) -> None:
        _check(cmn_plan_bind_adam(self.h, second_moments, stream), "cmn_plan_bind_adam")
        self._keep = (self._keep, second_moments)

    def allreduce_adam_step(self, alpha, beta1, beta2, eps, wd, t, mean_dest=CMN_MEAN_NONE, stream=None) -> None:
        _check(cmn_allreduce_adam_step(self.h, alpha, beta1, beta2, eps, wd, t, mean_dest, stream),
               "cmn_allreduce_adam_step")

    def allreduce_adam_step_range(self, tensor_begin, tensor_end, alpha, beta1, beta2, eps, wd, t,
                                  mean_dest=CMN_MEAN_NONE, stream=None) -> None:
        _check(cmn_allreduce_adam_step_range(self.h, tensor_begin, tensor_end, alpha, beta1, beta2, eps, wd, t,
                                             mean_dest, stream), "cmn_allreduce_adam_step_range")

    def adam(self, alpha, beta1, beta2, eps, wd, t, stream=None) -> None:
        _check(cmn_adam(self.h, alpha, beta1, beta2, eps, wd, t, stream), "cmn_adam")


# ------------------------------------------------------------------ device-memory plumbing for callers
def upload_tensors(arrays: Sequence[np.ndarray], misalign_elems: int = 0) -> List:
    """Each host array becomes its own device allocation (so that packing is a real
    gather).  ``misalign_elems`` > 0 returns views starting that many elements into a
    slightly larger allocation, to exercise unaligned base pointers."""
    import torch
    out = []
    for a in arrays:
        src = torch.from_numpy(np.ascontiguousarray(a))
        if misalign_elems:
            buf = torch.empty(src.numel() + misalign_elems, dtype=src.dtype, device="cuda")
            view = buf[misalign_elems:]
            view.copy_(src)
            out.append(view)
        else:
            out.append(src.to("cuda"))
    return out


def download_tensors(tensors: Sequence) -> List[np.ndarray]:
    return [t.detach().cpu().numpy() for t in tensors]
