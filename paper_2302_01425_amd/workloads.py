"""Seeded synthetic inputs for the five workloads.

This module only draws numbers.  It contains none of the method's arithmetic and is the one piece
of Python that both the tests of the CPU oracle and the callers of the HIP library may use, so
that both sides see the very same float32 buffers.

Generator: counter-based splitmix64 (stream position i of seed s is a pure function of (s, i)),
53-bit uniforms in (0, 1), Box-Muller for normals, inverse CDF for Laplace, then a cast to float32.

The shapes stand in for the paper's use sites (Sec. 6): a token-choice and an expert-choice
mixture-of-experts router (the paper routes k = 28 of n = 400 tokens for 32 experts), and magnitude
pruning that keeps 10 % of a weight matrix (k = ceil(n / 10), as in the paper's timing sweep).
None of the paper's datasets is used.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """Outputs start .. start+count-1 of the splitmix64 stream of ``seed`` (uint64)."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms strictly inside (0, 1)."""
    z = splitmix64(seed, start, count)
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, count: int, sigma: float = 1.0, chunk: int = 1 << 22) -> np.ndarray:
    """count float32 draws of N(0, sigma^2); element 2j and 2j+1 come from uniforms 2j, 2j+1."""
    out = np.empty(count, dtype=np.float32)
    pos = 0
    while pos < count:
        m = min(chunk, count - pos)
        m2 = m + (m & 1)
        u = uniform01(seed, pos, m2)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        ang = 2.0 * math.pi * u[1::2]
        z = np.empty(m2, dtype=np.float64)
        z[0::2] = r * np.cos(ang)
        z[1::2] = r * np.sin(ang)
        out[pos:pos + m] = (sigma * z[:m]).astype(np.float32)
        pos += m   # chunk is even, so only the last chunk can be odd
    return out


def laplace(seed: int, count: int, scale: float, chunk: int = 1 << 22) -> np.ndarray:
    """count float32 draws of Laplace(0, scale) by inverse CDF."""
    out = np.empty(count, dtype=np.float32)
    pos = 0
    while pos < count:
        m = min(chunk, count - pos)
        u = uniform01(seed, pos, m) - 0.5
        out[pos:pos + m] = (-scale * np.sign(u) * np.log1p(-2.0 * np.abs(u))).astype(np.float32)
        pos += m
    return out


def plant_ties(theta: np.ndarray, seed: int, frac: float = 0.05) -> np.ndarray:
    """Per row, overwrite round(frac * n) distinct positions with the (original) value of another,
    uniformly chosen position of the same row, creating exact duplicates."""
    rows, n = theta.shape
    m = int(round(frac * n))
    if m == 0 or n < 2:
        return theta
    u = uniform01(seed, 0, rows * n).reshape(rows, n)
    dst = np.argsort(u, axis=1, kind="stable")[:, :m]                  # m distinct destinations
    v = uniform01(seed ^ 0x5DEECE66D, 0, rows * m).reshape(rows, m)
    off = 1 + np.minimum((v * (n - 1)).astype(np.int64), n - 2)        # 1 .. n-1: never itself
    src = (dst + off) % n
    out = theta.copy()
    r = np.arange(rows)[:, None]
    out[r, dst] = theta[r, src]
    return out


@dataclass(frozen=True)
class Workload:
    name: str
    op: str            # "mask" (phi = identity) or "mag" (phi = x^2/2)
    rows: int
    n: int
    k: int
    p: float
    lam: float
    seed: int          # seed of the values; the tangent uses seed + 100
    dist: str          # "normal", "normal_ties", "laplace"
    scale: float

    def inputs(self):
        """(values, tangent), both float32 arrays of shape (rows, n)."""
        cnt = self.rows * self.n
        if self.dist == "laplace":
            x = laplace(self.seed, cnt, self.scale)
        else:
            x = normal(self.seed, cnt, self.scale)
        x = x.reshape(self.rows, self.n)
        if self.dist == "normal_ties":
            x = plant_ties(x, self.seed + 1000)
        t = normal(self.seed + 100, cnt, 1.0).reshape(self.rows, self.n)
        return np.ascontiguousarray(x), np.ascontiguousarray(t)


_N5 = 1 << 24

WORKLOADS = {
    # tiny batch the oracle finishes instantly
    "tiny": Workload("tiny", "mask", 64, 16, 2, 2.0, 1.0, 1, "normal", 1.0),
    # token-choice router: 16384 tokens x 64 experts, 5 % planted ties
    "moe_router": Workload("moe_router", "mask", 16384, 64, 2, 2.0, 0.5, 2, "normal_ties", 1.0),
    # smooth router: 32768 tokens x 128 experts, p = 4/3
    "moe_router_smooth": Workload("moe_router_smooth", "mask", 32768, 128, 8, 4.0 / 3.0, 1.0, 3,
                                  "normal", 2.0),
    # expert-choice router: 64 experts x 32768 tokens, rows span several workgroups
    "expert_choice": Workload("expert_choice", "mask", 64, 32768, 1024, 2.0, 0.1, 4, "normal", 1.0),
    # magnitude pruning of one flattened 4096 x 4096 layer, keep ceil(n / 10)
    "magnitude_pruning": Workload("magnitude_pruning", "mag", 1, _N5, -(-_N5 // 10), 2.0, 1e-3, 5,
                                  "laplace", 0.02),
    # the same layer with the p = 4/3 regulariser (not one of the five headline configurations:
    # the operator x p combination added after them)
    "magnitude_pruning_smooth": Workload("magnitude_pruning_smooth", "mag", 1, _N5, -(-_N5 // 10),
                                         4.0 / 3.0, 1e-3, 6, "laplace", 0.02),
}
