"""Helpers shared by the GPU parity tests: host <-> device marshalling and the comparison bars.

Bars (stated once, used everywhere):
  * integer, index and struct-of-integer results: bit-exact against the oracle;
  * floating point results: |gpu - ref| <= max(1e-4 * |ref|, 1e-3) element by element, where ref is
    the oracle's fp64 result on the same float32 inputs (relative 1e-4, absolute 1e-3 near zero);
  * min / max of floats are order independent and compared exactly.
"""
from __future__ import annotations

import numpy as np

import oracle
from ks_marshal import to_device, to_host  # noqa: F401  (re-exported for the tests)

RTOL, ATOL = 1e-4, 1e-3

# library (dtype, op) -> oracle (op, dt), numpy storage dtype, columns per element
KINDS = {
    ("i32", "sum"): ("sum", "i32", np.int32, 1), ("i32", "min"): ("min", "i32", np.int32, 1),
    ("i32", "max"): ("max", "i32", np.int32, 1),
    ("u32", "sum"): ("sum", "u32", np.uint32, 1), ("u32", "min"): ("min", "u32", np.uint32, 1),
    ("u32", "max"): ("max", "u32", np.uint32, 1),
    ("i64", "sum"): ("sum", "i64", np.int64, 1), ("i64", "min"): ("min", "i64", np.int64, 1),
    ("i64", "max"): ("max", "i64", np.int64, 1),
    ("u64", "sum"): ("sum", "u64", np.uint64, 1), ("u64", "min"): ("min", "u64", np.uint64, 1),
    ("u64", "max"): ("max", "u64", np.uint64, 1),
    ("f32", "sum"): ("sum", "f32", np.float32, 1), ("f32", "min"): ("min", "f32", np.float32, 1),
    ("f32", "max"): ("max", "f32", np.float32, 1),
    ("f64", "sum"): ("sum", "f64", np.float64, 1), ("f64", "min"): ("min", "f64", np.float64, 1),
    ("f64", "max"): ("max", "f64", np.float64, 1),
    ("affine_f32", "affine_compose"): ("affine", "f32", np.float32, 2),
    ("argmax_i32_cnt64", "argmax_count"): ("argmax", None, oracle.ARGMAX_DTYPE, 1),
    ("mat2_u32", "mat2_mul"): ("mat2", "u32", np.uint32, 4),
    ("quat_f32", "quat_mul"): ("quat", "f32", np.float32, 4),
    ("mat2_u64", "mat2_mul"): ("mat2", "u64", np.uint64, 4),                       # 32-byte elements
    ("range_i32_cnt32", "range_count"): ("range", None, oracle.RANGE_DTYPE, 1),     # 12-byte elements
}
FLOAT_TOL = {("f32", "sum"), ("f64", "sum"), ("affine_f32", "affine_compose"), ("quat_f32", "quat_mul")}

def random_input(dtype: str, op: str, n: int, seed: int) -> np.ndarray:
    """Generic seeded inputs for the (dtype, op) sweep (value ranges chosen so sums wrap and maxima tie)."""
    import ks_inputs
    rng = np.random.default_rng(seed)
    _, _, npdt, cols = KINDS[(dtype, op)]
    if dtype == "affine_f32":
        return ks_inputs.whole("affine", n, seed)
    if dtype == "argmax_i32_cnt64":
        x = ks_inputs.whole("argmax", n, seed)
        x["v"] = rng.integers(0, 50, size=n)          # many ties
        x["cnt"] = rng.integers(0, 1 << 40, size=n)
        return x
    if dtype == "mat2_u32":
        return ks_inputs.random_mat2(n, seed)
    if dtype == "quat_f32":
        return ks_inputs.random_unit_quats(n, seed)
    if dtype == "mat2_u64":
        return ks_inputs.random_mat2_wide(n, seed)
    if dtype == "range_i32_cnt32":
        return ks_inputs.random_ranges(n, seed)
    if np.issubdtype(npdt, np.integer):
        info = np.iinfo(npdt)
        return rng.integers(info.min, info.max, size=n, dtype=npdt, endpoint=True)
    if op == "sum":
        # Mixed signs at full amplitude: the running sum is a random walk (standard deviation
        # sqrt(n / 3), several thousand at the largest sizes) that keeps coming back to zero, where
        # only the absolute part of the bar is left.  tests/test_error_model.py derives what a scan
        # tiled like the GPU's can reach on exactly this kind of input.
        return rng.uniform(-1.0, 1.0, size=n).astype(npdt)
    return rng.normal(size=n).astype(npdt)


def reference(dtype: str, op: str, x: np.ndarray, inclusive: bool) -> np.ndarray:
    oop, odt, _, _ = KINDS[(dtype, op)]
    return oracle.scan(oop, odt, x, inclusive)


def float_bound(ref: np.ndarray) -> np.ndarray:
    """The floating point bar: relative RTOL, absolute ATOL where |ref| is below ATOL / RTOL."""
    return np.maximum(RTOL * np.abs(ref), ATOL)


def assert_matches(dtype: str, op: str, got: np.ndarray, ref: np.ndarray, what: str = "") -> float:
    """Apply the bar for this pair; returns the worst |err| / max(RTOL |ref|, ATOL) for float pairs, else 0."""
    if (dtype, op) in FLOAT_TOL:
        g = got.astype(np.float64).reshape(ref.shape)
        err = np.abs(g - ref)
        bound = float_bound(ref)
        worst = float(np.max(err / bound)) if err.size else 0.0
        if not worst <= 1.0:
            i = int(np.argmax(err / bound))
            raise AssertionError(f"{what}: float mismatch, worst ratio {worst:.3g} at flat index {i}: "
                                 f"gpu={g.reshape(-1)[i]!r} ref={ref.reshape(-1)[i]!r}")
        return worst
    g = got.reshape(ref.shape) if not got.dtype.names else got
    if g.tobytes() != ref.tobytes():
        if g.dtype.names:
            bad = np.nonzero(np.any([g[f] != ref[f] for f in g.dtype.names], axis=0))[0]
        else:
            bad = np.nonzero((g != ref).reshape(len(ref), -1).any(axis=1))[0]
        i = int(bad[0]) if len(bad) else -1
        raise AssertionError(f"{what}: {len(bad)} of {len(ref)} elements differ, first at {i}: "
                             f"gpu={g[i]!r} ref={ref[i]!r}")
    return 0.0
