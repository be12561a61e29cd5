"""Seeded synthetic workloads: parameter-list shapes and gradient/parameter values.

This module only *generates inputs*.  It holds none of the method's arithmetic
(no packing, summing, scaling or optimizer update) so that both the HIP path and
the CPU oracle can be fed the very same host arrays without sharing any code
that computes results.

The paper trains ResNet-50 on ImageNet with 32 images per GPU (Section 4.1) and
shows an MNIST MLP in Listing 1.  Neither dataset is needed here: the
aggregation + update path only ever sees per-layer gradient tensors, so
gradients are drawn from seeded normal distributions with the parameter-list
shapes of those models.

Configs (index = ``cfg``):
  1  MLP 784-256-256-10, K=2,   f32, grads N(0, 0.01),  lr .1  mu .9
  2  ResNet-50,          K=4,   f32, grads N(0, 1e-3/sqrt(fan_in))
  3  ResNet-50,          K=32,  f32, same             (headline)
  4  ResNet-50,          K=128, f16 storage, N(0,1e-3), 1 % of elements x100
  5  VGG-16,             K=16,  f32, N(0,1e-3), lr .01 mu .9 wd 5e-4
The second argument of every N(., .) is a standard deviation.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Sequence, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    fan_in: int  # in_ch*kh*kw (conv), in_features (fc), 1 for 1-D tensors

    @property
    def numel(self) -> int:
        return int(np.prod(self.shape, dtype=np.int64)) if self.shape else 1


def _conv(name, cout, cin, k):
    return TensorSpec(name, (cout, cin, k, k), cin * k * k)


def _vec(name, n):
    return TensorSpec(name, (n,), 1)


def _fc(name, nout, nin):
    return TensorSpec(name, (nout, nin), nin)


def mlp_list() -> List[TensorSpec]:
    """Listing 1's MNIST classifier shape: 784 -> 256 -> 256 -> 10 (W, b each)."""
    return [
        TensorSpec("l1.W", (784, 256), 784), _vec("l1.b", 256),
        TensorSpec("l2.W", (256, 256), 256), _vec("l2.b", 256),
        TensorSpec("l3.W", (256, 10), 256), _vec("l3.b", 10),
    ]


def resnet50_list() -> List[TensorSpec]:
    """Standard 224-px ResNet-50 in definition order: stem conv + BN, four
    stages of [3, 4, 6, 3] bottlenecks (1x1, 3x3, 1x1 x4, each followed by BN
    gamma/beta; the first block of a stage adds a projection conv + BN), then
    the 2048 -> 1000 classifier.  161 tensors, 25,557,032 elements."""
    out: List[TensorSpec] = [_conv("conv1.W", 64, 3, 7), _vec("bn1.gamma", 64), _vec("bn1.beta", 64)]
    cin = 64
    for s, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(blocks):
            p = f"res{s + 2}.{b}"
            out += [_conv(f"{p}.conv1.W", width, cin, 1), _vec(f"{p}.bn1.gamma", width), _vec(f"{p}.bn1.beta", width)]
            out += [_conv(f"{p}.conv2.W", width, width, 3), _vec(f"{p}.bn2.gamma", width), _vec(f"{p}.bn2.beta", width)]
            out += [_conv(f"{p}.conv3.W", 4 * width, width, 1), _vec(f"{p}.bn3.gamma", 4 * width), _vec(f"{p}.bn3.beta", 4 * width)]
            if b == 0:
                out += [_conv(f"{p}.proj.W", 4 * width, cin, 1), _vec(f"{p}.projbn.gamma", 4 * width), _vec(f"{p}.projbn.beta", 4 * width)]
            cin = 4 * width
    out += [_fc("fc.W", 1000, 2048), _vec("fc.b", 1000)]
    return out


def vgg16_list() -> List[TensorSpec]:
    """VGG-16: 13 3x3 convs (W, b) and 3 fully connected layers (W, b).
    32 tensors, 138,357,544 elements."""
    out: List[TensorSpec] = []
    cin = 3
    for i, cout in enumerate((64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512)):
        out += [_conv(f"conv{i + 1}.W", cout, cin, 3), _vec(f"conv{i + 1}.b", cout)]
        cin = cout
    for i, (nout, nin) in enumerate(((4096, 25088), (4096, 4096), (1000, 4096))):
        out += [_fc(f"fc{i + 1}.W", nout, nin), _vec(f"fc{i + 1}.b", nout)]
    return out


@dataclasses.dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    tensors: Tuple[TensorSpec, ...]
    K: int            # worker replicas
    n_chunks: int     # ring chunks
    grad_dtype: str   # "f32" | "f16" | "bf16" | "i8s"  (storage type; bf16 as uint16 bit patterns; "i8s" =
                      # int8 + per-chunk scales, produced from the f32 draws by quantise_i8)
    grad_std: float
    per_layer_fan_in_scale: bool
    outlier_frac: float
    outlier_scale: float
    lr: float
    mu: float
    wd: float
    param_std: float = 0.05
    align_bytes: int = 256

    @property
    def numel(self) -> List[int]:
        return [t.numel for t in self.tensors]

    @property
    def N(self) -> int:
        return sum(self.numel)


def config(cfg: int) -> Config:
    if cfg == 1:
        return Config(1, "mlp_k2_f32", tuple(mlp_list()), 2, 2, "f32", 0.01, False, 0.0, 1.0, 0.1, 0.9, 0.0)
    if cfg == 2:
        return Config(2, "resnet50_k4_f32", tuple(resnet50_list()), 4, 4, "f32", 1e-3, True, 0.0, 1.0, 0.1, 0.9, 0.0)
    if cfg == 3:
        return Config(3, "resnet50_k32_f32", tuple(resnet50_list()), 32, 32, "f32", 1e-3, True, 0.0, 1.0, 0.1, 0.9, 0.0)
    if cfg == 4:
        return Config(4, "resnet50_k128_f16", tuple(resnet50_list()), 128, 128, "f16", 1e-3, False, 0.01, 100.0, 0.1, 0.9, 0.0)
    if cfg == 5:
        return Config(5, "vgg16_k16_f32", tuple(vgg16_list()), 16, 16, "f32", 1e-3, False, 0.0, 1.0, 0.01, 0.9, 5e-4)
    raise ValueError(f"unknown config {cfg}")


def custom_config(numel: Sequence[int], K: int, n_chunks: int, grad_dtype: str = "f32", *, cfg: int = 90,
                  grad_std: float = 1e-2, lr: float = 0.1, mu: float = 0.9, wd: float = 0.0,
                  outlier_frac: float = 0.0, align_bytes: int = 256) -> Config:
    """A small ad-hoc tensor list (ragged sizes, zero-sized tensors, ...) for edge-case tests."""
    specs = tuple(TensorSpec(f"t{i}", (int(n),), 1) for i, n in enumerate(numel))
    return Config(cfg, f"custom{cfg}", specs, K, n_chunks, grad_dtype, grad_std, False, outlier_frac, 100.0,
                  lr, mu, wd, 0.05, align_bytes)


# ----------------------------------------------------------------------------
# value generators
# ----------------------------------------------------------------------------

def grad_seed(cfg: int, step: int, k: int) -> int:
    return 1_000_000 * cfg + 1_000 * step + k


def param_seed(cfg: int) -> int:
    return 1_000_000 * cfg + 999_999


def _split(flat: np.ndarray, numel: Sequence[int]) -> List[np.ndarray]:
    out, o = [], 0
    for n in numel:
        out.append(flat[o:o + n])
        o += n
    return out


def _bf16_bits(x: np.ndarray) -> np.ndarray:
    """Quantise finite float32 inputs to bfloat16 bit patterns (nearest, ties to even)."""
    u = x.view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def gen_grads(c: Config, step: int, k: int) -> List[np.ndarray]:
    """Replica ``k``'s per-layer gradients for iteration ``step`` (list of 1-D
    arrays in list order; dtype float32 or float16 per ``c.grad_dtype``)."""
    rng = np.random.Generator(np.random.PCG64(grad_seed(c.cfg, step, k)))
    numel = c.numel
    flat = rng.standard_normal(c.N, dtype=np.float32)
    o = 0
    for t, n in zip(c.tensors, numel):
        std = c.grad_std / math.sqrt(t.fan_in) if c.per_layer_fan_in_scale else c.grad_std
        flat[o:o + n] *= np.float32(std)
        o += n
    if c.outlier_frac > 0.0:
        mask = rng.random(c.N, dtype=np.float32) < np.float32(c.outlier_frac)
        flat[mask] *= np.float32(c.outlier_scale)
    if c.grad_dtype == "f16":
        return _split(flat.astype(np.float16), numel)  # round-to-nearest-even
    if c.grad_dtype == "bf16":
        return _split(_bf16_bits(flat), numel)         # uint16 bit patterns
    return _split(flat, numel)                         # "f32", and "i8s" before quantise_i8


def quantise_i8(tensors: Sequence[np.ndarray], chunk_elems: int, n_chunks: int):
    """Producer-side quantisation of one replica's float32 gradients for the int8 storage format:
    per ring chunk (chunk_elems consecutive elements of the tight concatenation) one float32 scale
    = max|g| / 127 (1 if the chunk is all zero or padding) and q = rint(g / scale) in [-127, 127].
    Returns (list of int8 tensors, float32 array of n_chunks scales)."""
    flat = np.concatenate([np.asarray(t, np.float32).reshape(-1) for t in tensors]) if tensors else np.zeros(0, np.float32)
    q = np.zeros(flat.size, np.int8)
    scales = np.ones(n_chunks, np.float32)
    for c in range(n_chunks):
        seg = flat[c * chunk_elems:(c + 1) * chunk_elems]
        if seg.size and np.abs(seg).max() > 0:
            scales[c] = np.float32(np.abs(seg).max()) / np.float32(127.0)
            q[c * chunk_elems:c * chunk_elems + seg.size] = np.clip(np.rint(seg / scales[c]), -127, 127).astype(np.int8)
    return _split(q, [np.asarray(t).size for t in tensors]), scales


def gen_grads_f32_unquantised(c: Config, step: int, k: int) -> List[np.ndarray]:
    """The float32 values *before* fp16 rounding (same draws as ``gen_grads``)."""
    return gen_grads(dataclasses.replace(c, grad_dtype="f32"), step, k)


def gen_params(c: Config) -> List[np.ndarray]:
    rng = np.random.Generator(np.random.PCG64(param_seed(c.cfg)))
    flat = rng.standard_normal(c.N, dtype=np.float32) * np.float32(c.param_std)
    return _split(flat, c.numel)


def gen_velocity(c: Config) -> List[np.ndarray]:
    return _split(np.zeros(c.N, dtype=np.float32), c.numel)
