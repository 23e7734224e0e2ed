"""Seeded synthetic inputs for the scan workloads.

This module only draws random numbers and lays them out; it holds none of the
scan's arithmetic, and it is the only code shared by the CPU oracle's tests and
the GPU tests / benchmark.

Recipe (identical for every consumer): ``numpy.random.default_rng(seed)``,
drawn in fixed chunks of CHUNK = 2**24 elements in index order, so the sequence
for a given (workload, n) never depends on who asks or how it is consumed.

Workloads (they stand in for the paper's unstated Float32/Float64 arrays of
1e6..1e9 elements, Sec. VII; the paper uses no public data set):

  int32_sum    inclusive sum,  int32,   uniform integers in [-100, 100],  seed 0
  f32_sum      inclusive sum,  float32, uniform [0, 1),                   seed 1
  u64_exsum    exclusive sum,  uint64,  uniform integers in [0, 2**32),   seed 2
  affine       inclusive affine-map composition, (a, b) float32 pairs,
               a uniform [0.99, 1.01], b uniform [-1, 1],                 seed 3
  argmax       inclusive running arg-max with count, 16-byte struct
               {int32 v, int32 idx, int64 cnt}: v uniform in [0, 2**20),
               idx = position, cnt = 1,                                    seed 4
  f64_sum      inclusive sum,  float64, uniform [0, 1),                   seed 5
               (the paper's other benchmarked element type, Tables II and IV)
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator

import numpy as np

CHUNK = 1 << 24

ARGMAX_DTYPE = np.dtype([("v", "<i4"), ("idx", "<i4"), ("cnt", "<i8")])


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # library dtype name
    op: str             # library operator name
    inclusive: bool
    n: int              # size the headline configuration is quoted on
    seed: int
    elem_bytes: int


WORKLOADS = {
    "int32_sum": Workload("int32_sum", "i32", "sum", True, 1 << 20, 0, 4),
    "f32_sum": Workload("f32_sum", "f32", "sum", True, 1 << 28, 1, 4),
    "u64_exsum": Workload("u64_exsum", "u64", "sum", False, 1 << 27, 2, 8),
    "affine": Workload("affine", "affine_f32", "affine_compose", True, 1 << 26, 3, 8),
    "argmax": Workload("argmax", "argmax_i32_cnt64", "argmax_count", True, 1 << 30, 4, 16),
    "f64_sum": Workload("f64_sum", "f64", "sum", True, 1 << 27, 5, 8),
    # uint8 codes, uniform over 0 .. 255: the 8-bit types of the paper's mapreduce benchmark (reductions only)
    "u8_codes": Workload("u8_codes", "u8", "sum", True, 10 ** 9, 6, 1),
    # 16-bit floats as bit patterns, values uniform in (-1, 1): running sums with float32 arithmetic
    "bf16_sum": Workload("bf16_sum", "bf16", "sum", True, 1 << 29, 7, 2),
    "f16_sum": Workload("f16_sum", "f16", "sum", True, 1 << 29, 8, 2),
}

ARGMAX_SWEEP = [1 << k for k in range(10, 31, 2)]   # 2^10 .. 2^30 in powers of 4


def _draw(name: str, rng: np.random.Generator, start: int, m: int) -> np.ndarray:
    if name == "int32_sum":
        return rng.integers(-100, 101, size=m, dtype=np.int32)
    if name == "f32_sum":
        return rng.random(size=m, dtype=np.float32)
    if name == "f64_sum":
        return rng.random(size=m, dtype=np.float64)
    if name == "u64_exsum":
        return rng.integers(0, 1 << 32, size=m, dtype=np.uint64)
    if name == "u8_codes":
        return rng.integers(0, 256, size=m, dtype=np.uint8)
    if name == "bf16_sum":      # float32 values cut to their upper 16 bits
        return (rng.uniform(-1.0, 1.0, size=m).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    if name == "f16_sum":
        return rng.uniform(-1.0, 1.0, size=m).astype(np.float16).view(np.uint16)
    if name == "affine":
        out = np.empty((m, 2), dtype=np.float32)
        out[:, 0] = rng.uniform(0.99, 1.01, size=m).astype(np.float32)
        out[:, 1] = rng.uniform(-1.0, 1.0, size=m).astype(np.float32)
        return out
    if name == "argmax":
        out = np.empty(m, dtype=ARGMAX_DTYPE)
        out["v"] = rng.integers(0, 1 << 20, size=m, dtype=np.int32)
        out["idx"] = np.arange(start, start + m, dtype=np.int64).astype(np.int32)
        out["cnt"] = 1
        return out
    raise KeyError(name)


def chunks(name: str, n: int | None = None, seed: int | None = None) -> Iterator[np.ndarray]:
    """Yield the workload's input in order, CHUNK elements at a time."""
    w = WORKLOADS[name]
    n = w.n if n is None else int(n)
    rng = np.random.default_rng(w.seed if seed is None else seed)
    start = 0
    while start < n:
        m = min(CHUNK, n - start)
        yield _draw(name, rng, start, m)
        start += m


def whole(name: str, n: int | None = None, seed: int | None = None) -> np.ndarray:
    """The whole input as one array (use only when it fits host memory)."""
    parts = list(chunks(name, n, seed))
    if not parts:
        w = WORKLOADS[name]
        return _draw(name, np.random.default_rng(w.seed), 0, 0)
    return parts[0] if len(parts) == 1 else np.concatenate(parts)


def random_mat2(n: int, seed: int) -> np.ndarray:
    """n random 2x2 uint32 matrices, row-major (n, 4): an exact non-commutative test type."""
    return np.random.default_rng(seed).integers(0, 1 << 32, size=(n, 4), dtype=np.uint32)


def random_mat2_wide(n: int, seed: int) -> np.ndarray:
    """n random 2x2 uint64 matrices, row-major (n, 4): the 32-byte exact non-commutative test type."""
    return np.random.default_rng(seed).integers(0, 1 << 64, size=(n, 4), dtype=np.uint64)


RANGE_DTYPE = np.dtype([("lo", "<i4"), ("hi", "<i4"), ("cnt", "<u4")])


def random_ranges(n: int, seed: int) -> np.ndarray:
    """n elements {x, x, c} of the 12-byte range-with-count type: x a random walk (new minima and maxima
    keep appearing), c a random count so that the sums wrap."""
    rng = np.random.default_rng(seed)
    x = np.cumsum(rng.integers(-1000, 1001, size=n)).astype(np.int32)
    out = np.empty(n, dtype=RANGE_DTYPE)
    out["lo"], out["hi"] = x, x
    out["cnt"] = rng.integers(0, 1 << 32, size=n, dtype=np.uint32)
    return out


def random_codes(n: int, seed: int, skew: float = 0.0) -> np.ndarray:
    """n uint8 codes, drawn in fixed chunks so that any prefix of a longer draw is the shorter draw.
    skew = 0: uniform over 0 .. 255 (as UnitFloat8 levels: mixed signs, the sum a random walk
    around zero); skew > 0: that share of the codes is moved into the upper half (a sum that grows)."""
    out = np.empty(n, np.uint8)
    for i, at in enumerate(range(0, n, CHUNK)):
        rng = np.random.default_rng([seed, 77, i])
        m = min(CHUNK, n - at)
        c = rng.integers(0, 256, size=CHUNK, dtype=np.uint8)[:m]
        if skew > 0.0:
            up = rng.random(CHUNK)[:m] < skew
            c = np.where(up, c | np.uint8(0x80), c)
        out[at:at + m] = c
    return out


def random_half_bits(kind: str, n: int, seed: int, spikes: bool = True) -> np.ndarray:
    """n finite 16-bit floats as uint16 bit patterns, values in (-1, 1), with `spikes` a tenth of them
    up to +-64: kind "bf16" (the upper 16 bits of a float32, truncated) or "f16" (IEEE binary16, rounded)."""
    rng = np.random.default_rng([seed, 99])
    v = rng.uniform(-1.0, 1.0, size=n).astype(np.float32)
    if spikes:
        v *= np.where(rng.random(n) < 0.1, np.float32(64.0), np.float32(1.0))
    if kind == "bf16":
        return (v.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    if kind == "f16":
        return v.astype(np.float16).view(np.uint16)
    raise KeyError(kind)


def random_unit_quats(n: int, seed: int) -> np.ndarray:
    """n unit quaternions (w, x, y, z) as float32 (n, 4)."""
    q = np.random.default_rng(seed).normal(size=(n, 4))
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return q.astype(np.float32)
