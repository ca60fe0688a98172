"""Seeded synthetic inputs shaped like the paper's ResNet workloads.

This module holds NO arithmetic of the method (no pooling, inflation or
convolution): only layer shapes, a counter-based random generator, the value
recipe and storage-type rounding.  It serves both the CPU oracle's tests and the
HIP path so that both see bit-identical inputs.

Recipe (experiments section: ResNet18 on ImageNet; the data itself is not
needed, only tensors with the same shape and structure):
  X  = ReLU(N(0,1))          post-ReLU conv input, about half exact zeros
  dY ~ N(0, dy_std)          dy_std = 1 (0.1 for the deep small-spatial stress)
  W  ~ N(0, 2/(C*R*S))       Kaiming-normal, fan-in
  b  = small N(0, 0.01)      so that a dropped bias term is visible in parity
every tensor drawn from numpy's Philox generator keyed by
(base seed, config name, layer name, tensor name), then rounded to the storage
type (float32, or bfloat16 by round-to-nearest-even).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class LayerSpec:
    name: str
    N: int
    C: int      # input channels
    K: int      # output channels
    H: int
    W: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1
    k: int = 2  # pooling factor of the saved input (1 = uncompressed)
    dtype: str = BF16
    dy_std: float = 1.0

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def dw_flops(self) -> int:
        """Executed multiply-adds of the weight gradient, times two."""
        return 2 * self.N * self.P * self.Q * self.K * self.C * self.R * self.S

    def with_k(self, k: int) -> "LayerSpec":
        return replace(self, k=k)


def _c3(name, N, C, K, H, stride=1, **kw):
    return LayerSpec(name, N, C, K, H, H, 3, 3, stride, 1, **kw)


def _c1(name, N, C, K, H, stride=1, **kw):
    return LayerSpec(name, N, C, K, H, H, 1, 1, stride, 0, **kw)


def _resnet18_imagenet(N: int, k: int) -> List[LayerSpec]:
    # Conv layers of ResNet18 behind the (uncompressed) stem: architecture figure
    # and per-layer memory table.  One representative of each distinct shape.
    return [
        _c3("l1.3x3_64_64@56", N, 64, 64, 56, k=k),
        _c3("l2.3x3s2_64_128@56", N, 64, 128, 56, 2, k=k),
        _c1("l2.1x1s2_64_128@56", N, 64, 128, 56, 2, k=k),
        _c3("l2.3x3_128_128@28", N, 128, 128, 28, k=k),
        _c3("l3.3x3s2_128_256@28", N, 128, 256, 28, 2, k=k),
        _c1("l3.1x1s2_128_256@28", N, 128, 256, 28, 2, k=k),
        _c3("l3.3x3_256_256@14", N, 256, 256, 14, k=k),
        _c3("l4.3x3s2_256_512@14", N, 256, 512, 14, 2, k=k),
        _c1("l4.1x1s2_256_512@14", N, 256, 512, 14, 2, k=k),
        _c3("l4.3x3_512_512@7", N, 512, 512, 7, k=k),
    ]


def _resnet50_imagenet(N: int, k: int) -> List[LayerSpec]:
    out: List[LayerSpec] = []
    cin, hin = 64, 56
    for st, (mid, cout, h) in enumerate([(64, 256, 56), (128, 512, 28), (256, 1024, 14),
                                         (512, 2048, 7)], start=1):
        s = 1 if st == 1 else 2
        out += [
            _c1(f"s{st}.b0.1x1_{cin}_{mid}@{hin}", N, cin, mid, hin, k=k),
            _c3(f"s{st}.b0.3x3s{s}_{mid}_{mid}@{hin}", N, mid, mid, hin, s, k=k),
            _c1(f"s{st}.b0.1x1_{mid}_{cout}@{h}", N, mid, cout, h, k=k),
            _c1(f"s{st}.b0.down1x1s{s}_{cin}_{cout}@{hin}", N, cin, cout, hin, s, k=k),
            _c1(f"s{st}.b1.1x1_{cout}_{mid}@{h}", N, cout, mid, h, k=k),
            _c3(f"s{st}.b1.3x3_{mid}_{mid}@{h}", N, mid, mid, h, k=k),
        ]
        cin, hin = cout, h
    return out


def configs() -> Dict[str, List[LayerSpec]]:
    """The five workload configurations, by name."""
    cfg: Dict[str, List[LayerSpec]] = {}
    cfg["cfg1_single_fp32"] = [LayerSpec("conv3x3_16_16@32", 8, 16, 16, 32, 32, dtype=F32)]
    cfg["cfg2_resnet18_cifar"] = [
        _c3(f"3x3_{c}_{c}@{h}", 128, c, c, h) for c, h in ((64, 32), (128, 16), (256, 8), (512, 4))
    ]
    cfg["cfg3_resnet50_imagenet"] = _resnet50_imagenet(64, 2)
    for k in (1, 2, 4):
        cfg[f"cfg4_resnet18_imagenet_k{k}"] = _resnet18_imagenet(128, k)
    cfg["cfg5_deep_small_spatial"] = [
        _c3("3x3_512_512@14", 256, 512, 512, 14, dy_std=0.1),
        _c3("3x3_512_512@7", 256, 512, 512, 7, dy_std=0.1),
    ]
    return cfg


# ----------------------------------------------------------------------------
# storage-type rounding (type conversion only)

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array holding bfloat16-representable values (RNE)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array of bfloat16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not bfloat16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == BF16 else a


# ----------------------------------------------------------------------------
# seeded generation

def _rng(seed: int, config: str, layer: str, tensor: str) -> np.random.Generator:
    digest = hashlib.sha256(f"{seed}|{config}|{layer}|{tensor}".encode()).digest()
    key = int.from_bytes(digest[:16], "little")
    return np.random.Generator(np.random.Philox(key=key))


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def make_inputs(spec: LayerSpec, config: str = "adhoc", seed: int = 0,
                tensors=("X", "W", "b", "dY")) -> Dict[str, np.ndarray]:
    """float32 arrays already rounded to spec.dtype (so fp64 copies of them are
    exactly what the device sees)."""
    out: Dict[str, np.ndarray] = {}
    if "X" in tensors:
        x = _normal(_rng(seed, config, spec.name, "X"), (spec.N, spec.C, spec.H, spec.W), 1.0)
        np.maximum(x, 0.0, out=x)
        out["X"] = to_storage(x, spec.dtype)
    if "W" in tensors:
        std = float(np.sqrt(2.0 / (spec.C * spec.R * spec.S)))
        out["W"] = to_storage(_normal(_rng(seed, config, spec.name, "W"),
                                      (spec.K, spec.C, spec.R, spec.S), std), spec.dtype)
    if "b" in tensors:
        out["b"] = to_storage(_normal(_rng(seed, config, spec.name, "b"), (spec.K,), 0.01), spec.dtype)
    if "dY" in tensors:
        out["dY"] = to_storage(_normal(_rng(seed, config, spec.name, "dY"),
                                       (spec.N, spec.K, spec.P, spec.Q), spec.dy_std), spec.dtype)
    return out
