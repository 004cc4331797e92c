"""Seeded, counter-based random inputs shared by the oracle tests and the GPU tests.

This module holds no arithmetic of the fusion method: it only produces the
synthetic inputs and weights both sides consume.  Every draw is a pure
function of (seed, stream, element index), so any slice of any tensor can be
regenerated independently of the order in which tensors are requested.

Generator: the splitmix64 finaliser applied to a 64-bit counter (public
definition by Steele, Lea, Flood), 53-bit uniforms, Box-Muller normals.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def raw_u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit words of stream `stream` under `seed`, starting at element `offset`."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]) + _GOLD * np.uint64(2 * stream + 1))[0]
        ctr = np.arange(offset, offset + n, dtype=np.uint64)
        return _mix(key + _GOLD * (ctr + np.uint64(1)))


def uniform01(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """float64 uniforms in [0, 1) with 53 random bits."""
    return (raw_u64(seed, stream, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(seed, stream, shape, lo=0.0, hi=1.0) -> np.ndarray:
    n = int(np.prod(shape, dtype=np.int64))
    return (lo + (hi - lo) * uniform01(seed, stream, n)).reshape(shape)


def normal(seed, stream, shape, mean=0.0, std=1.0) -> np.ndarray:
    """Box-Muller on two independent sub-streams; one normal per counter value."""
    n = int(np.prod(shape, dtype=np.int64))
    u1 = 1.0 - uniform01(seed, 2 * stream + 1_000_003, n)  # (0, 1]
    u2 = uniform01(seed, 2 * stream + 1_000_004, n)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (mean + std * z).reshape(shape)


def integers(seed, stream, shape, lo, hi) -> np.ndarray:
    """int64 uniform in [lo, hi)."""
    n = int(np.prod(shape, dtype=np.int64))
    r = raw_u64(seed, stream, n) % np.uint64(hi - lo)
    return (r.astype(np.int64) + lo).reshape(shape)


# ---- storage rounding (inputs are rounded once to the config's storage type) ----

def round_to(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to storage dtype (RNE) and return them widened back
    to float32 (f32/f16/bf16 values are all exactly representable in float32)."""
    if dtype in ("i32", "i64"):
        return np.rint(a).astype(np.int64)
    if dtype == "f32":
        return a.astype(np.float32)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        f = a.astype(np.float32)
        u = f.view(np.uint32).astype(np.uint64)
        lsb = (u >> np.uint64(16)) & np.uint64(1)
        u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
        return u.astype(np.uint32).view(np.float32).reshape(f.shape)
    raise ValueError(dtype)
