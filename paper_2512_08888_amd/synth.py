"""Seeded synthetic inputs for the rotation-convolution workloads.

This module holds no arithmetic of the method itself: it only produces the
tensors (images, base filter banks, upstream gradients) that both the CPU
oracle and the HIP path are fed with, so the two sides see bit-identical
inputs on any machine.  It imports neither of them.

Generator: a counter-based SplitMix64 (one 64-bit hash per element index), so
a tensor depends only on (seed, element index) and never on the order in which
tensors are drawn.  Normals come from Box-Muller on two hashed uniforms, in
fp64, and are rounded to fp32 once at the end.

The workloads stand in for the paper's UAV segmentation data (Sec. V-B: RGB
images scaled to [0,1), integer class masks) and for the activations of its
UNet layers (Sec. V-A); none of the paper's datasets is reproduced.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _hash64(seed: int, idx: np.ndarray) -> np.ndarray:
    """SplitMix64 output function applied to seed + (idx+1)*golden."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (idx.astype(np.uint64) + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """n fp64 uniforms in [0,1) for element indices offset .. offset+n-1."""
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for s in range(0, n, step):
        e = min(n, s + step)
        idx = np.arange(offset + s, offset + e, dtype=np.uint64)
        out[s:e] = (_hash64(seed, idx) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return out


def normal01(seed: int, n: int) -> np.ndarray:
    """n fp64 standard normals (Box-Muller on uniforms 2i and 2i+1)."""
    out = np.empty(n, dtype=np.float64)
    step = 1 << 21
    for s in range(0, n, step):
        e = min(n, s + step)
        idx = np.arange(s, e, dtype=np.uint64)
        u1 = (_hash64(seed, idx * np.uint64(2)) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        u2 = (_hash64(seed, idx * np.uint64(2) + np.uint64(1)) >> np.uint64(11)).astype(np.float64) * (
            1.0 / 9007199254740992.0
        )
        out[s:e] = np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * math.pi * u2)
    return out


def randint(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi] (inclusive)."""
    span = hi - lo + 1
    idx = np.arange(n, dtype=np.uint64)
    return (lo + (_hash64(seed, idx) >> np.uint64(33)).astype(np.int64) % span).astype(np.int64)


@dataclass(frozen=True)
class LayerConfig:
    """One rotation-convolution layer workload (problem statement of Sec. III)."""

    name: str
    N: int
    Cin: int
    H: int
    W: int
    Cout: int
    k: int = 3
    R: int = 4
    mode: str = "exact90"          # "exact90" | "steerable" | "bilinear" | "p4m"
    stride: int = 1
    pad: int = 1
    pool_group: Optional[int] = None  # None -> R (one pooled map per filter)
    x_dist: str = "uniform"        # "uniform" U[0,1) | "absnormal" |N(0,1)| | "normal"
    angles_deg: Optional[Sequence[float]] = None
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.R if self.pool_group is None else self.pool_group

    @property
    def B(self) -> int:
        return 2 if self.mode == "steerable" else 1

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Cpool(self) -> int:
        return self.Cout * (self.R // self.G)

    def angles(self) -> np.ndarray:
        if self.angles_deg is not None:
            return np.asarray(self.angles_deg, dtype=np.float64)
        return np.arange(self.R, dtype=np.float64) * (360.0 / self.R)


# The three single-layer workloads the benchmark description names.
C1 = LayerConfig("C1", N=1, Cin=3, H=64, W=64, Cout=8, R=4, x_dist="uniform", seed=1000)
C2 = LayerConfig("C2", N=8, Cin=64, H=256, W=256, Cout=64, R=4, x_dist="absnormal", seed=2000)
C3 = LayerConfig("C3", N=4, Cin=128, H=128, W=128, Cout=128, R=16, mode="bilinear", x_dist="absnormal", seed=3000)

# The first layer (RGB image -> 64 filters) of the UNet-shaped stacks of configurations 4 and 5, as a layer of its own.
C4_ENC0A = LayerConfig("C4_enc0a", N=4, Cin=3, H=512, W=512, Cout=64, R=4, x_dist="uniform", seed=4100)
C5_ENC0A = LayerConfig("C5_enc0a", N=2, Cin=3, H=512, W=512, Cout=64, R=16, mode="bilinear", x_dist="uniform", seed=5100)

# ... and the second one (64 -> 64 channels at full resolution), the shallow R = 16 layer of configuration 5.
C5_ENC0B = LayerConfig("C5_enc0b", N=2, Cin=64, H=512, W=512, Cout=64, R=16, mode="bilinear", x_dist="absnormal", seed=5200)

CONFIGS = {"C1": C1, "C2": C2, "C3": C3, "C4_enc0a": C4_ENC0A, "C5_enc0a": C5_ENC0A, "C5_enc0b": C5_ENC0B}


def make_x(cfg: LayerConfig) -> np.ndarray:
    n = cfg.N * cfg.Cin * cfg.H * cfg.W
    if cfg.x_dist == "uniform":
        v = uniform01(cfg.seed + 1, n)
    elif cfg.x_dist == "absnormal":
        v = np.abs(normal01(cfg.seed + 1, n))
    elif cfg.x_dist == "normal":
        v = normal01(cfg.seed + 1, n)
    else:
        raise ValueError(cfg.x_dist)
    return v.astype(np.float32).reshape(cfg.N, cfg.Cin, cfg.H, cfg.W)


def make_w(cfg: LayerConfig) -> np.ndarray:
    """He-normal base bank(s): std = sqrt(2 / (Cin k^2)).  Shape [B,Cout,Cin,k,k]."""
    n = cfg.B * cfg.Cout * cfg.Cin * cfg.k * cfg.k
    std = math.sqrt(2.0 / (cfg.Cin * cfg.k * cfg.k))
    return (normal01(cfg.seed + 2, n) * std).astype(np.float32).reshape(cfg.B, cfg.Cout, cfg.Cin, cfg.k, cfg.k)


def make_g(cfg: LayerConfig) -> np.ndarray:
    """Upstream gradient w.r.t. the pooled output, N(0,1).  Shape [N,Cpool,Ho,Wo]."""
    n = cfg.N * cfg.Cpool * cfg.Ho * cfg.Wo
    return normal01(cfg.seed + 3, n).astype(np.float32).reshape(cfg.N, cfg.Cpool, cfg.Ho, cfg.Wo)


def make_dy(cfg: LayerConfig) -> np.ndarray:
    """Dense upstream gradient w.r.t. the unpooled output, N(0,1).  [N,Cout*R,Ho,Wo]."""
    n = cfg.N * cfg.Cout * cfg.R * cfg.Ho * cfg.Wo
    return normal01(cfg.seed + 4, n).astype(np.float32).reshape(cfg.N, cfg.Cout * cfg.R, cfg.Ho, cfg.Wo)


def make_idx(cfg: LayerConfig) -> np.ndarray:
    """A valid random orientation-index map (for backward tests that need none
    of the forward): idx[n, co*(R/G)+g, y, x] is a member of pool group g."""
    ng = cfg.R // cfg.G
    n = cfg.N * cfg.Cpool * cfg.Ho * cfg.Wo
    j = randint(cfg.seed + 5, n, 0, cfg.G - 1).reshape(cfg.N, cfg.Cout, ng, cfg.Ho, cfg.Wo)
    g = np.arange(ng, dtype=np.int64).reshape(1, 1, ng, 1, 1)
    return (j * ng + g).astype(np.uint8).reshape(cfg.N, cfg.Cpool, cfg.Ho, cfg.Wo)


# --- exact-arithmetic ("dyadic") variants -----------------------------------
# Values on coarse binary grids, so that every partial sum of the forward and of
# the input gradient is exactly representable in fp32 whatever the summation
# order; results of the two sides must then agree bit for bit, ties included.

def make_x_dyadic(cfg: LayerConfig) -> np.ndarray:
    n = cfg.N * cfg.Cin * cfg.H * cfg.W
    return (randint(cfg.seed + 11, n, 0, 15).astype(np.float32) / 16.0).reshape(cfg.N, cfg.Cin, cfg.H, cfg.W)


def make_w_dyadic(cfg: LayerConfig) -> np.ndarray:
    n = cfg.B * cfg.Cout * cfg.Cin * cfg.k * cfg.k
    return (randint(cfg.seed + 12, n, -16, 16).astype(np.float32) / 32.0).reshape(
        cfg.B, cfg.Cout, cfg.Cin, cfg.k, cfg.k
    )


def make_g_dyadic(cfg: LayerConfig) -> np.ndarray:
    n = cfg.N * cfg.Cpool * cfg.Ho * cfg.Wo
    return (randint(cfg.seed + 13, n, -32, 32).astype(np.float32) / 8.0).reshape(cfg.N, cfg.Cpool, cfg.Ho, cfg.Wo)
