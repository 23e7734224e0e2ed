"""TEST INFRASTRUCTURE: sequential CPU oracle for the device-wide scan.

Nothing in the product path may import this package.  It wraps the plain-C
left fold in ``scan_oracle.c`` (built with gcc into ``liboracle_scan.so``) and
adds a pure-Python fold over arbitrary Python objects for tiny cases.

Definition followed (paper, Sec. II-C, scan; Sec. V-B first sentence):
``out[i] = in[0] op ... op in[i]`` (inclusive) or ``in[0] op ... op in[i-1]``
with ``out[0] = identity`` (exclusive), ``op`` associative and not necessarily
commutative, the accumulated value always being the left operand.

``mapreduce`` (paper, Sec. II-C and V-A) is the same fold taken to the end:
``op(f(src[1]), ..., f(src[n]))``, written as the left fold of the mapped
elements, accumulated value on the left.

Every function here is pinned by tests/test_oracle_pins.py and
tests/test_oracle_mapreduce_pins.py to closed forms, library special cases,
exact sums and brute force over every parenthesisation (and, for commutative
operators, every order of the elements); none is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scan_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_scan.so")

ARGMAX_DTYPE = np.dtype([("v", "<i4"), ("idx", "<i4"), ("cnt", "<i8")])
RANGE_DTYPE = np.dtype([("lo", "<i4"), ("hi", "<i4"), ("cnt", "<u4")])     # 12 bytes


def build(force: bool = False) -> str:
    """Compile scan_oracle.c with gcc (no HIP, no shared headers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
             "-ffp-contract=off", _SRC, "-o", _LIB])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


# name -> (C symbol, input numpy dtype, output numpy dtype, words per element in, out,
#          accumulator ctype fields)
_SCALAR_CTYPES = {
    "i32": ctypes.c_int32, "u32": ctypes.c_uint32, "i64": ctypes.c_int64, "u64": ctypes.c_uint64,
    "f32": ctypes.c_float, "f64": ctypes.c_double,
}
_NP = {"i32": np.int32, "u32": np.uint32, "i64": np.int64, "u64": np.uint64,
       "f32": np.float32, "f64": np.float64}


def _scalar_state(acc_ctype):
    class State(ctypes.Structure):
        _fields_ = [("acc", acc_ctype), ("started", ctypes.c_int)]
    return State


class _AffineState(ctypes.Structure):
    _fields_ = [("a", ctypes.c_double), ("b", ctypes.c_double), ("started", ctypes.c_int)]


class _ArgmaxElem(ctypes.Structure):
    _fields_ = [("v", ctypes.c_int32), ("idx", ctypes.c_int32), ("cnt", ctypes.c_int64)]


class _ArgmaxState(ctypes.Structure):
    _fields_ = [("acc", _ArgmaxElem), ("started", ctypes.c_int)]


class _Mat2State(ctypes.Structure):
    _fields_ = [("acc", ctypes.c_uint32 * 4), ("started", ctypes.c_int)]


class _Mat2WideState(ctypes.Structure):
    _fields_ = [("acc", ctypes.c_uint64 * 4), ("started", ctypes.c_int)]


class _RangeState(ctypes.Structure):
    _fields_ = [("acc", ctypes.c_int32 * 3), ("started", ctypes.c_int)]


class _QuatState(ctypes.Structure):
    _fields_ = [("q", ctypes.c_double * 4), ("started", ctypes.c_int)]


def _scalar_entry(op: str, dt: str):
    """(symbol, in dtype, out dtype, state class) for a scalar (op, dtype) pair."""
    if op == "sum":
        acc = {"i32": ctypes.c_uint32, "u32": ctypes.c_uint32, "i64": ctypes.c_uint64,
               "u64": ctypes.c_uint64, "f32": ctypes.c_double, "f64": ctypes.c_longdouble}[dt]
        out = {"f32": np.float64}.get(dt, _NP[dt])
    elif op in ("min", "max"):
        acc = _SCALAR_CTYPES[dt]
        out = _NP[dt]
    else:
        raise KeyError(op)
    return f"oracle_{op}_{dt}", _NP[dt], out, _scalar_state(acc)


class ScanStream:
    """A scan fed in chunks; the running value is carried between feed() calls.

    kind is one of: ("sum"|"min"|"max", "i32"|"u32"|"i64"|"u64"|"f32"|"f64"),
    ("affine", "f32"), ("argmax", None), ("mat2", "u32"), ("mat2", "u64"), ("range", None),
    ("quat", "f32").
    Shapes: scalars (n,), affine (n, 2), quat (n, 4), mat2 (n, 4) uint32 or uint64,
    argmax (n,) of ARGMAX_DTYPE, range (n,) of RANGE_DTYPE.
    """

    def __init__(self, op: str, dt: str | None, inclusive: bool = True):
        self.op, self.dt, self.inclusive = op, dt, bool(inclusive)
        lib = _load()
        if op in ("sum", "min", "max"):
            sym, self.in_dtype, self.out_dtype, state_cls = _scalar_entry(op, dt)
            self.width = 1
        elif op == "affine":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_affine_f32", np.float32, np.float64, _AffineState, 2
        elif op == "argmax":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_argmax", ARGMAX_DTYPE, ARGMAX_DTYPE, _ArgmaxState, 1
        elif op == "mat2" and dt == "u64":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_mat2_u64", np.uint64, np.uint64, _Mat2WideState, 4
        elif op == "mat2":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_mat2_u32", np.uint32, np.uint32, _Mat2State, 4
        elif op == "range":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_range_i32", RANGE_DTYPE, RANGE_DTYPE, _RangeState, 1
        elif op == "quat":
            sym, self.in_dtype, self.out_dtype, state_cls, self.width = \
                "oracle_quat_f32", np.float32, np.float64, _QuatState, 4
        else:
            raise KeyError(op)
        self._fn = getattr(lib, sym)
        self._fn.restype = None
        self._fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                             ctypes.c_void_p]
        self._state = state_cls()
        ctypes.memset(ctypes.byref(self._state), 0, ctypes.sizeof(self._state))

    def feed(self, chunk: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(chunk, dtype=self.in_dtype)
        if self.width > 1:
            assert x.ndim == 2 and x.shape[1] == self.width, x.shape
        else:
            assert x.ndim == 1, x.shape
        n = x.shape[0]
        out = np.empty(x.shape, dtype=self.out_dtype)
        if n:
            self._fn(x.ctypes.data, out.ctypes.data, n, int(self.inclusive),
                     ctypes.addressof(self._state))
        return out


def scan(op: str, dt: str | None, x: np.ndarray, inclusive: bool = True) -> np.ndarray:
    """One-shot sequential scan of a whole array (see ScanStream for kinds)."""
    return ScanStream(op, dt, inclusive).feed(x)


def apply_map(name: str, x: np.ndarray, kind: str | None = None) -> np.ndarray:
    """The element-wise map f of the map-fused scan ``scan(f, op, src)`` (paper Sec. IV-A).

    identity: x;  square: x * x (integers wrap in their own width; float32 inputs are squared in
    float64, where the product of two float32 values is exact);  abs: |x| (the most negative integer
    maps to itself);  nonzero: 1 where x != 0 else 0, in x's type.

    Two maps change the type, f: T -> S of the paper's Sec. II-C, and take uint8 codes only:
    unit_float8: code c stands for level c of 256 evenly spaced levels from -1 to +1 (paper
    Sec. VII-B, the 8-bit type of the mapreduce benchmark), (2c - 255) / 255, promoted to float32:
    the float32 nearest to that rational (float64 division, then one rounding to float32; the
    quotient of two small integers is far from any float32 tie, which the pins check code by code);
    widen64: the code as a uint64, so that a sum of bytes cannot wrap.
    widen_f32 takes uint16 bit patterns and `kind` ("bf16" or "f16") and gives the float32 of the same value.
    """
    x = np.asarray(x)
    if name == "widen_f32":
        # 16-bit floats stored as uint16 bit patterns, promoted to float32 (every such value is a
        # float32 exactly): "bf16" = the upper half of a float32's bits, "f16" = IEEE binary16
        if x.dtype != np.uint16 or kind not in ("bf16", "f16"):
            raise TypeError("map 'widen_f32' takes uint16 bit patterns of kind 'bf16' or 'f16'")
        if kind == "bf16":
            return (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return x.view(np.float16).astype(np.float32)
    if name in ("unit_float8", "widen64"):
        if x.dtype != np.uint8:
            raise TypeError(f"map {name!r} takes uint8 codes")
        if name == "widen64":
            return x.astype(np.uint64)
        return ((2.0 * x.astype(np.float64) - 255.0) / 255.0).astype(np.float32)
    if name == "identity":
        return x
    if name == "square":
        if np.issubdtype(x.dtype, np.floating):
            y = x.astype(np.float64)
            return y * y
        with np.errstate(over="ignore"):
            u = x.view(np.dtype(f"u{x.dtype.itemsize}"))
            return (u * u).view(x.dtype)
    if name == "abs":
        if np.issubdtype(x.dtype, np.floating):
            return np.abs(x)
        with np.errstate(over="ignore"):
            return np.where(x < 0, (0 - x.view(np.dtype(f"u{x.dtype.itemsize}"))).view(x.dtype), x)
    if name == "nonzero":
        return (x != 0).astype(x.dtype)
    raise ValueError(f"unknown map {name!r}")


def mapped_scan(map_name: str, op: str, dt: str, x: np.ndarray, inclusive: bool = True) -> np.ndarray:
    """out[i] = f(x[0]) op ... op f(x[i]) (paper Sec. IV-A): the map, then the plain sequential scan."""
    y = apply_map(map_name, x)
    if y.dtype == np.float64 and dt == "f32":
        dt = "f64"   # squares of float32 values, held exactly in float64
    return scan(op, dt, np.ascontiguousarray(y), inclusive)


def identity_of(op: str, dt: str | None):
    """The operator's identity in the oracle's output type (what an empty reduction returns)."""
    if op == "sum":
        return (np.float64 if dt in ("f32", "f64") else _NP[dt])(0)
    if op in ("min", "max"):
        t = _NP[dt]
        if np.issubdtype(t, np.floating):
            return t(np.inf if op == "min" else -np.inf)
        info = np.iinfo(t)
        return t(info.max if op == "min" else info.min)
    if op == "affine":
        return np.array([1.0, 0.0])
    if op == "argmax":
        return np.array([(np.iinfo(np.int32).min, np.iinfo(np.int32).max, 0)], dtype=ARGMAX_DTYPE)[0]
    if op == "mat2":
        return np.array([1, 0, 0, 1], dtype=np.uint64 if dt == "u64" else np.uint32)
    if op == "range":
        return np.array([(np.iinfo(np.int32).max, np.iinfo(np.int32).min, 0)], dtype=RANGE_DTYPE)[0]
    if op == "quat":
        return np.array([1.0, 0.0, 0.0, 0.0])
    raise KeyError(op)


def mapreduce(map_name: str, op: str, dt: str | None, x: np.ndarray, chunk: int = 1 << 22):
    """op(f(x[0]), f(x[1]), ..., f(x[n-1])) as one sequential left fold (paper Sec. II-C, mapreduce;
    Sec. V-A), the accumulated value always on the left; the identity for an empty input.

    The fold is the scan's own (the same C routine run to the end of the input, fed in chunks, the
    running value carried in its state); what comes back is the last running value, in the oracle's
    output type: float64 for float32 / float64 sums, affine maps and quaternions, the element type
    (the map's result type, where the map changes it) for everything else.  The paper asks for a commutative operator here; the left fold is also
    defined for the non-commutative ones, and that is what is returned for them.
    """
    x = np.asarray(x)
    n = x.shape[0]
    if dt == "u8":
        # bytes: sums only.  unit_float8 -> a float32 sum, widen64 -> a uint64 sum; with no map the
        # sum stays in the element type, i.e. modulo 2^8 (what UInt8 + UInt8 is), and the exact sum
        # reduced modulo 2^8 is that value whatever the order of the additions.
        if op != "sum":
            raise KeyError((op, dt))
        if map_name == "identity":
            return np.uint8(int(mapreduce("widen64", "sum", "u8", x, chunk)) & 0xFF)
        dt = {"unit_float8": "f32", "widen64": "u64"}[map_name]
    kind = None
    if dt in ("bf16", "f16"):
        # 16-bit floats: reduced after promotion to float32 (sum, min, max), nothing else
        if map_name != "widen_f32" or op not in ("sum", "min", "max"):
            raise KeyError((map_name, op, dt))
        kind, dt = dt, "f32"
    if n == 0:
        return identity_of(op, dt)
    if kind is not None:
        stream = ScanStream(op, dt, True)
        last = None
        for at in range(0, n, chunk):
            last = stream.feed(np.ascontiguousarray(apply_map(map_name, x[at:at + chunk], kind)))[-1]
        return last
    probe = apply_map(map_name, x[:1])
    if probe.dtype == np.float64 and dt == "f32":
        dt = "f64"   # squares of float32 values, held exactly in float64
    stream = ScanStream(op, dt, True)
    last = None
    for at in range(0, n, chunk):
        last = stream.feed(np.ascontiguousarray(apply_map(map_name, x[at:at + chunk])))[-1]
    return last


def fold_scan(op, xs, inclusive=True, identity=None):
    """Pure-Python left fold over arbitrary objects: the definition itself.

    ``op(earlier, later)``; exclusive needs ``identity``.  For tiny cases and
    for operators the C file does not carry.
    """
    out = []
    if inclusive:
        acc = None
        for i, x in enumerate(xs):
            acc = x if i == 0 else op(acc, x)
            out.append(acc)
    else:
        if identity is None:
            raise ValueError("exclusive scan needs the operator's identity")
        acc = identity
        for x in xs:
            out.append(acc)
            acc = op(acc, x)
    return out
