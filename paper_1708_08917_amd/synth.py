"""Seeded synthetic inputs for the block-circulant layer workloads.

This module only draws numbers.  It holds none of the method's arithmetic
(no circulant expansion, no FFT, no layer math), so that the CPU oracle and
the HIP path can both be fed from it without sharing any of their own code.

Every element is a pure function of (seed, tensor_id, element index): a
counter-based 64-bit mixer gives a uniform in [0, 1); normals come from the
Box-Muller transform of two such uniforms.  Values are rounded once to fp32;
both sides then start from exactly the same fp32 buffers.

Workload shapes and value distributions follow the five layer configurations
of this build (FC 1024x1024/k=16, FC 4096x4096/k=64, the 9216-4096-4096
classifier head/k=128, the 3x3 CONV 256->256/k=64 and the FC 16384x16384/k=256
forward+backward case); `N(0, v)` is read as a normal with *variance* v.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 1708089170

# tensor ids: one stream per tensor of a configuration
T_W, T_X, T_BIAS, T_DY, T_W2, T_BIAS2 = 0, 1, 2, 3, 4, 5

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_C_SEED = np.uint64(0x9E3779B97F4A7C15)
_C_TENSOR = np.uint64(0xD1B54A32D192ED03)
_C_INDEX = np.uint64(0x94D049BB133111EB)
_MIX1 = np.uint64(0xBF58476D1CE4E5B9)
_MIX2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _MIX1
        z = (z ^ (z >> np.uint64(27))) * _MIX2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, tensor_id: int, n: int, stream: int = 0) -> np.ndarray:
    """n doubles in [0, 1), element e = f(seed, tensor_id, stream, e)."""
    with np.errstate(over="ignore"):
        idx = np.arange(n, dtype=np.uint64)
        key = (np.uint64(seed) * _C_SEED) ^ (np.uint64(tensor_id * 2 + stream + 1) * _C_TENSOR)
        z = _mix64(_mix64(key + idx * _C_INDEX) + idx)
    return (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed: int, tensor_id: int, shape, lo: float, hi: float) -> np.ndarray:
    n = int(np.prod(shape))
    u = uniform01(seed, tensor_id, n)
    return (lo + (hi - lo) * u).astype(np.float32).reshape(shape)


def normal(seed: int, tensor_id: int, shape, variance: float) -> np.ndarray:
    n = int(np.prod(shape))
    u1 = uniform01(seed, tensor_id, n, stream=0)
    u2 = uniform01(seed, tensor_id, n, stream=1)
    r = np.sqrt(-2.0 * np.log1p(-u1))
    z = r * np.cos(2.0 * math.pi * u2)
    return (math.sqrt(variance) * z).astype(np.float32).reshape(shape)


def small_integers(seed: int, tensor_id: int, shape, lo: int = -8, hi: int = 8) -> np.ndarray:
    """Integers in [lo, hi] as fp32: every product and sum of a layer stays exact."""
    n = int(np.prod(shape))
    u = uniform01(seed, tensor_id, n)
    return np.floor(lo + (hi - lo + 1) * u).astype(np.float32).reshape(shape)


@dataclass
class FcConfig:
    name: str
    n_in: int
    n_out: int
    k: int
    batch: int
    bias: bool
    relu: bool
    x_lo: float = -1.0
    x_hi: float = 1.0
    index: int = 0
    p: int = field(init=False)
    q: int = field(init=False)

    def __post_init__(self):
        assert self.n_in % self.k == 0 and self.n_out % self.k == 0
        self.p = self.n_out // self.k
        self.q = self.n_in // self.k


@dataclass
class ConvConfig:
    name: str
    N: int
    C_in: int
    C_out: int
    H: int
    W: int
    r: int
    stride: int
    pad: int
    k: int
    index: int = 0

    @property
    def p(self):
        return self.C_out // self.k

    @property
    def q(self):
        return self.C_in // self.k


CFG1 = FcConfig("fc1024_k16_b1", 1024, 1024, 16, 1, bias=False, relu=False, index=0)
CFG2 = FcConfig("fc4096_k64_b64", 4096, 4096, 64, 64, bias=True, relu=True, index=1)
CFG3_L1 = FcConfig("head_fc9216x4096_k128_b256", 9216, 4096, 128, 256, bias=True, relu=True,
                   x_lo=0.0, x_hi=1.0, index=2)
CFG3_L2 = FcConfig("head_fc4096x4096_k128_b256", 4096, 4096, 128, 256, bias=True, relu=True,
                   x_lo=0.0, x_hi=1.0, index=2)
CFG4 = ConvConfig("conv3x3_c256_28x28_k64_n32", 32, 256, 256, 28, 28, 3, 1, 1, 64, index=3)
CFG5 = FcConfig("fc16384_k256_b1024", 16384, 16384, 256, 1024, bias=False, relu=False, index=4)


def fc_inputs(cfg: FcConfig, seed_offset: int = 0, second_layer: bool = False, batch: int | None = None):
    """(w[p][q][k], x[B][n_in], bias[n_out] or None) as fp32 arrays."""
    seed = BASE_SEED + cfg.index + 1000 * seed_offset
    B = cfg.batch if batch is None else batch
    w = normal(seed, T_W2 if second_layer else T_W, (cfg.p, cfg.q, cfg.k), 1.0 / cfg.n_in)
    x = uniform(seed, T_X, (B, cfg.n_in), cfg.x_lo, cfg.x_hi)
    b = normal(seed, T_BIAS2 if second_layer else T_BIAS, (cfg.n_out,), 0.01) if cfg.bias else None
    return w, x, b


def fc_upstream_grad(cfg: FcConfig, seed_offset: int = 0, batch: int | None = None) -> np.ndarray:
    seed = BASE_SEED + cfg.index + 1000 * seed_offset
    B = cfg.batch if batch is None else batch
    return uniform(seed, T_DY, (B, cfg.n_out), -1.0, 1.0)


def conv_inputs(cfg: ConvConfig, seed_offset: int = 0, batch: int | None = None):
    """(w[r][r][p][q][k], x[N][C_in][H][W]) as fp32 arrays (offset-major weights)."""
    seed = BASE_SEED + cfg.index + 1000 * seed_offset
    N = cfg.N if batch is None else batch
    w = normal(seed, T_W, (cfg.r, cfg.r, cfg.p, cfg.q, cfg.k), 2.0 / (cfg.r * cfg.r * cfg.C_in))
    x = uniform(seed, T_X, (N, cfg.C_in, cfg.H, cfg.W), -1.0, 1.0)
    return w, x


def conv_upstream_grad(cfg: ConvConfig, seed_offset: int = 0, batch: int | None = None):
    """dL/da [N][C_out][Ho][Wo], Uniform[-1, 1] (the CONV counterpart of fc_upstream_grad)."""
    seed = BASE_SEED + cfg.index + 1000 * seed_offset
    N = cfg.N if batch is None else batch
    Ho, Wo = cfg.H + 2 * cfg.pad - cfg.r + 1, cfg.W + 2 * cfg.pad - cfg.r + 1
    return uniform(seed, T_DY, (N, cfg.C_out, Ho, Wo), -1.0, 1.0)

