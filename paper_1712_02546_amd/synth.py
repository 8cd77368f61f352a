"""Seeded synthetic inputs for the benchmark and parity configurations.

Only shapes, seeds and random draws live here -- none of the convolution's
arithmetic -- so that the HIP path and the CPU oracle can be fed the same bytes.
Shapes follow the paper's CIFAR-10 network (32x32x3 inputs, two 5x5 convolution
layers with pooling of stride 2 in between, 500 and 1500 kernels in the largest
network, batch 128: Section 5.2) plus one larger-image pair of layers.  The
dataset itself is not used; value distributions stand in for images (uniform
[0,1)), rectified activations (max(N(0,1),0)) and upstream gradients (N(0,1)).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 171202546


@dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int          # seed family
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    k0: int = 0
    k1: int = -1
    x_dist: str = "uniform"      # "uniform" -> U[0,1); "relu" -> max(N(0,1),0)
    w_std: float = 0.05

    @property
    def slice(self) -> tuple[int, int]:
        return (self.k0, self.K if self.k1 < 0 else self.k1)

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def flops_per_pass(self) -> int:
        k0, k1 = self.slice
        return 2 * self.N * (k1 - k0) * self.P * self.Q * self.C * self.R * self.S

    def with_slice(self, k0: int, k1: int) -> "LayerConfig":
        return replace(self, k0=k0, k1=k1)


CONFIGS = {
    "cfg1": LayerConfig("cfg1", 1, N=8, C=3, H=32, W=32, K=16, R=5, S=5),
    "cfg2": LayerConfig("cfg2", 2, N=128, C=3, H=32, W=32, K=500, R=5, S=5),
    "cfg3": LayerConfig("cfg3", 3, N=128, C=500, H=14, W=14, K=1500, R=5, S=5, x_dist="relu", w_std=0.01),
    # one device's share of cfg3: same tensors (same seed family), kernels 500..999
    "cfg4": LayerConfig("cfg4", 3, N=128, C=500, H=14, W=14, K=1500, R=5, S=5, k0=500, k1=1000,
                        x_dist="relu", w_std=0.01),
    "cfg5a": LayerConfig("cfg5a", 5, N=64, C=3, H=224, W=224, K=96, R=11, S=11, stride=4, pad=2),
    "cfg5b": LayerConfig("cfg5b", 6, N=64, C=96, H=27, W=27, K=256, R=5, S=5, pad=2, x_dist="relu",
                         w_std=0.01),
}


def _rng(cfg: LayerConfig, which: int) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * cfg.index + which)


def make_x(cfg: LayerConfig) -> np.ndarray:
    g = _rng(cfg, 0)
    shape = (cfg.N, cfg.C, cfg.H, cfg.W)
    if cfg.x_dist == "uniform":
        return g.random(shape, dtype=np.float32)
    if cfg.x_dist == "relu":
        return np.maximum(g.standard_normal(shape, dtype=np.float32), np.float32(0))
    raise ValueError(cfg.x_dist)


def make_w(cfg: LayerConfig) -> np.ndarray:
    g = _rng(cfg, 1)
    return (g.standard_normal((cfg.K, cfg.C, cfg.R, cfg.S), dtype=np.float32) * np.float32(cfg.w_std))


def make_dy(cfg: LayerConfig) -> np.ndarray:
    g = _rng(cfg, 2)
    return g.standard_normal((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=np.float32)


def make_inputs(cfg: LayerConfig):
    """(x, w, dy) as float32 numpy arrays, full-layer tensors."""
    return make_x(cfg), make_w(cfg), make_dy(cfg)


def random_layer(seed: int, N, C, H, W, K, R, S, stride=1, pad=0, k0=0, k1=-1) -> LayerConfig:
    """An ad-hoc shape for edge-case tests; seeded by ``seed``."""
    return LayerConfig(f"adhoc{seed}", 100 + seed, N, C, H, W, K, R, S, stride, pad, k0, k1,
                       x_dist="relu", w_std=0.05)


# ---- bfloat16 as bit patterns (upper half of an fp32, round to nearest even) ----
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bfloat16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))
