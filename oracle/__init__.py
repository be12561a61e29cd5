"""CPU oracle (test infrastructure, NOT the product path).

Thin ctypes wrapper over ``cmn_oracle.c`` plus the step-by-step composition of
the whole aggregation + update iteration.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; it imports
nothing from the HIP package and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cmn_oracle.c")
_LIB = os.path.join(_HERE, "libcmn_oracle.so")

F32, F16, BF16, I8S = 0, 1, 2, 3
_DT = {"f32": F32, "f16": F16, "bf16": BF16, "i8s": I8S, F32: F32, F16: F16, BF16: BF16, I8S: I8S}
_NP = {F32: np.float32, F16: np.float16, BF16: np.uint16, I8S: np.int8}   # bfloat16 travels as raw 16-bit patterns


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: one rounding per operation, OpenMP over chunks."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # the mutation test points this at a deliberately broken copy to show the pins catch it
        L = ctypes.CDLL(os.environ.get("CMN_ORACLE_LIB_FOR_MUTATION_TEST") or build())
        i64p = ctypes.POINTER(ctypes.c_int64)
        vpp = ctypes.POINTER(ctypes.c_void_p)
        fp = ctypes.POINTER(ctypes.c_float)
        L.orc_half_bits_to_float.restype = ctypes.c_float
        L.orc_half_bits_to_float.argtypes = [ctypes.c_uint16]
        L.orc_geometry.restype = ctypes.c_int
        L.orc_geometry.argtypes = [ctypes.c_int, i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   i64p, i64p, i64p, i64p]
        L.orc_pack.restype = None
        L.orc_pack.argtypes = [ctypes.c_int, i64p, vpp, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]
        L.orc_direct_fold.restype = None
        L.orc_direct_fold.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, vpp, ctypes.c_int,
                                      ctypes.c_int, vpp, fp]
        L.orc_ring_allreduce.restype = ctypes.c_int
        L.orc_ring_allreduce.argtypes = [ctypes.c_int, ctypes.c_int64, vpp]
        L.orc_scale.restype = None
        L.orc_scale.argtypes = [ctypes.c_int64, fp, ctypes.c_int, fp]
        L.orc_unpack.restype = None
        L.orc_unpack.argtypes = [ctypes.c_int, i64p, fp, vpp]
        L.orc_momentum_sgd.restype = None
        L.orc_momentum_sgd.argtypes = [ctypes.c_int64, fp, fp, fp, ctypes.c_float, ctypes.c_float,
                                       ctypes.c_float]
        L.orc_bf16_bits_to_float.restype = ctypes.c_float
        L.orc_bf16_bits_to_float.argtypes = [ctypes.c_uint16]
        L.orc_float_to_bf16_bits.restype = ctypes.c_uint16
        L.orc_float_to_bf16_bits.argtypes = [ctypes.c_float]
        L.orc_float_to_bf16_array.restype = None
        L.orc_float_to_bf16_array.argtypes = [ctypes.c_int64, fp, ctypes.c_void_p]
        L.orc_float_to_half_bits.restype = ctypes.c_uint16
        L.orc_float_to_half_bits.argtypes = [ctypes.c_float]
        L.orc_float_to_half_array.restype = None
        L.orc_float_to_half_array.argtypes = [ctypes.c_int64, fp, ctypes.c_void_p]
        L.orc_adam_lr.restype = ctypes.c_float
        L.orc_adam_lr.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int]
        L.orc_adam.restype = None
        L.orc_adam.argtypes = [ctypes.c_int64, fp, fp, fp, fp] + [ctypes.c_float] * 5
        L.orc_max_threads.restype = ctypes.c_int
        L.orc_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def _i64(a: Sequence[int]):
    arr = np.ascontiguousarray(a, dtype=np.int64)
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _ptrs(arrays: Sequence[np.ndarray]):
    p = (ctypes.c_void_p * max(1, len(arrays)))()
    for i, a in enumerate(arrays):
        assert a.flags["C_CONTIGUOUS"]
        p[i] = a.ctypes.data
    return p


def _fp(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def max_threads() -> int:
    return int(lib().orc_max_threads())


def half_bits_to_float(h: int) -> np.float32:
    return np.float32(lib().orc_half_bits_to_float(int(h) & 0xFFFF))


class Geometry:
    def __init__(self, numel: Sequence[int], n_chunks: int, align_bytes: int = 256, dtype="f32"):
        self.numel, npp = _i64(numel)
        self.T = len(self.numel)
        self.C = int(n_chunks)
        self.dtype = _DT[dtype]
        self.off = np.zeros(self.T + 1, dtype=np.int64)
        N, ce, L = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        rc = lib().orc_geometry(self.T, npp, self.C, int(align_bytes), self.dtype,
                                self.off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                ctypes.byref(N), ctypes.byref(ce), ctypes.byref(L))
        if rc != 0:
            raise ValueError("invalid geometry arguments")
        self.N, self.chunk_elems, self.L = N.value, ce.value, L.value


def pack(geo: Geometry, tensors: Sequence[np.ndarray]) -> np.ndarray:
    """S1 for one replica: T tensors -> packed[L] (same dtype), padding zero."""
    npdt = _NP[geo.dtype]
    ts = [np.ascontiguousarray(t, dtype=npdt).reshape(-1) for t in tensors]
    assert [t.size for t in ts] == list(geo.numel)
    out = np.empty(geo.L, dtype=npdt)
    _, npp = _i64(geo.numel)
    lib().orc_pack(geo.T, npp, _ptrs(ts), geo.dtype, geo.L, out.ctypes.data)
    return out


def direct_fold(geo: Geometry, packed: Sequence[np.ndarray], ring_rotate: int = 1,
                scales: Sequence[np.ndarray] = None) -> np.ndarray:
    """S2 by definition: K packed buffers -> float32 sum[L], fixed fold order.
    scales[k] (float32, one per ring chunk) is required for int8 storage."""
    K = len(packed)
    for b in packed:
        assert b.dtype == _NP[geo.dtype] and b.size == geo.L
    assert (scales is not None) == (geo.dtype == I8S)
    if scales is not None:
        scales = [np.ascontiguousarray(s, dtype=np.float32) for s in scales]
        assert len(scales) == K and all(s.size == geo.C for s in scales)
    out = np.empty(geo.L, dtype=np.float32)
    lib().orc_direct_fold(K, geo.C, geo.chunk_elems, _ptrs(packed), geo.dtype, int(ring_rotate),
                          _ptrs(scales) if scales is not None else None, _fp(out))
    return out


def ring_allreduce(chunk_elems: int, bufs: List[np.ndarray]) -> None:
    """S2 by simulation: K float32 rank buffers of K*chunk_elems, overwritten in place."""
    K = len(bufs)
    for b in bufs:
        assert b.dtype == np.float32 and b.size == K * chunk_elems and b.flags["C_CONTIGUOUS"]
    if lib().orc_ring_allreduce(K, int(chunk_elems), _ptrs(bufs)) != 0:
        raise MemoryError


def decode_to_f32(a: np.ndarray) -> np.ndarray:
    """Element-wise binary16 -> binary32 through the oracle's own bit-level decoder."""
    if a.dtype == np.float32:
        return a.copy()
    bits = a.view(np.uint16).reshape(-1)
    out = np.empty(bits.size, dtype=np.float32)
    f = lib().orc_half_bits_to_float
    for i, h in enumerate(bits):          # slow on purpose; used on small inputs only
        out[i] = f(int(h))
    return out.reshape(a.shape)


def scale(total: np.ndarray, K: int) -> np.ndarray:
    out = np.empty_like(total)
    lib().orc_scale(total.size, _fp(total), int(K), _fp(out))
    return out


def unpack(geo: Geometry, gbar: np.ndarray) -> List[np.ndarray]:
    outs = [np.empty(int(n), dtype=np.float32) for n in geo.numel]
    _, npp = _i64(geo.numel)
    lib().orc_unpack(geo.T, npp, _fp(gbar), _ptrs(outs))
    return outs


def momentum_sgd(g: np.ndarray, p: np.ndarray, v: np.ndarray, lr: float, mu: float, wd: float) -> None:
    """S5 on one tensor, p and v updated in place."""
    assert g.size == p.size == v.size
    lib().orc_momentum_sgd(g.size, _fp(g), _fp(p), _fp(v), float(lr), float(mu), float(wd))


def float_to_half(a: np.ndarray) -> np.ndarray:
    """binary32 -> binary16, round to nearest even, through the oracle's own encoder."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().orc_float_to_half_array(a.size, _fp(a.reshape(-1)), out.ctypes.data)
    return out.view(np.float16)


def float_to_bf16(a: np.ndarray) -> np.ndarray:
    """binary32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().orc_float_to_bf16_array(a.size, _fp(a.reshape(-1)), out.ctypes.data)
    return out


def bf16_bits_to_float(b: int) -> np.float32:
    return np.float32(lib().orc_bf16_bits_to_float(int(b) & 0xFFFF))


def adam_lr(alpha: float, beta1: float, beta2: float, t: int) -> float:
    return float(lib().orc_adam_lr(alpha, beta1, beta2, int(t)))


def adam(g: np.ndarray, p: np.ndarray, m: np.ndarray, v: np.ndarray, alpha: float, beta1: float, beta2: float,
         eps: float, wd: float, t: int) -> None:
    """Adam on one tensor at iteration t (1-based); p, m, v updated in place."""
    assert g.size == p.size == m.size == v.size
    lib().orc_adam(g.size, _fp(g), _fp(p), _fp(m), _fp(v), adam_lr(alpha, beta1, beta2, t), float(beta1),
                   float(beta2), float(eps), float(wd))


def mean_gradients(grads: Sequence[Sequence[np.ndarray]], numel: Sequence[int], n_chunks: int, *, dtype="f32",
                   align_bytes: int = 256, ring_rotate: int = 1, scales=None) -> List[np.ndarray]:
    """S1..S4: pack, fold, scale, unpack -> the T averaged gradient tensors (float32)."""
    K = len(grads)
    geo = Geometry(numel, n_chunks, align_bytes, dtype)
    packed = [pack(geo, grads[k]) for k in range(K)]
    return unpack(geo, scale(direct_fold(geo, packed, ring_rotate, scales), K))


def allreduce_step(grads: Sequence[Sequence[np.ndarray]], params: List[np.ndarray], vels: List[np.ndarray],
                   n_chunks: int, lr: float, mu: float, wd: float, *, dtype="f32", align_bytes: int = 256,
                   ring_rotate: int = 1, scales=None) -> List[np.ndarray]:
    """The whole iteration, step after step with every intermediate materialised:
    pack each of the K replicas, fold, scale, unpack, MomentumSGD per tensor.
    ``grads[k][t]``; params/vels are updated in place; returns the mean gradients."""
    K = len(grads)
    geo = Geometry([p.size for p in params], n_chunks, align_bytes, dtype)
    packed = [pack(geo, grads[k]) for k in range(K)]
    total = direct_fold(geo, packed, ring_rotate, scales)
    gbar = scale(total, K)
    mean = unpack(geo, gbar)
    for t in range(geo.T):
        momentum_sgd(mean[t], params[t], vels[t], lr, mu, wd)
    return mean
