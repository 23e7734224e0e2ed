"""ks_scan: device-wide inclusive / exclusive scan for AMD MI355X (gfx950).

Thin Python binding over the C-ABI library ``libks_scan.so`` (declared in
``include/ks_scan.h``).  It only marshals arguments: PyTorch supplies device
memory and the stream, every step of the scan runs in the library's HIP
kernels.  There is no CPU or PyTorch fallback: if the library is missing the
import of this package fails.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported first so that the library binds to the HIP runtime torch already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libks_scan.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python paper_2603_18695_amd/build.py` "
        "(hipcc, --offload-arch=gfx950). There is no fallback path.")

_lib = ctypes.CDLL(LIB_PATH)

KS_OK = 0
KS_ERR_INVALID_ARG, KS_ERR_UNSUPPORTED, KS_ERR_MISALIGNED, KS_ERR_OVERLAP = -1, -2, -3, -4
KS_ERR_WORKSPACE, KS_ERR_HIP, KS_ERR_TIMEOUT = -5, -6, -7

DTYPES = {"i32": 0, "u32": 1, "i64": 2, "u64": 3, "f32": 4, "f64": 5, "affine_f32": 6,
          "argmax_i32_cnt64": 7, "mat2_u32": 8, "quat_f32": 9, "mat2_u64": 10, "range_i32_cnt32": 11, "u8": 12, "bf16": 13, "f16": 14}
OPS = {"sum": 0, "min": 1, "max": 2, "affine_compose": 3, "argmax_count": 4, "mat2_mul": 5, "quat_mul": 6,
       "range_count": 7}
ALGOS = {"auto": 0, "lookback": 1, "reduce_then_scan": 2}
MAPS = {"identity": 0, "square": 1, "abs": 2, "nonzero": 3, "unit_float8": 4, "widen64": 5, "widen_f32": 6}

EXPORTS = ["ks_scan", "ks_scan_seeded", "ks_scan_static", "ks_mapreduce", "ks_mapreduce_result_bytes", "ks_release_scratch", "ks_scan_pair", "ks_mapreduce_pair", "ks_pair_elem_bytes", "ks_scan_map", "ks_scan_strided", "ks_map_supported", "ks_scan_temp_bytes", "ks_scan_with_temp",
           "ks_scan_check", "ks_pair_supported",
           "ks_elem_bytes", "ks_set_option", "ks_get_option", "ks_copy", "ks_status_string",
           "ks_last_hip_error", "ks_version"]

_vp, _sz, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_lib.ks_scan.argtypes = [_i, _i, _i, _vp, _vp, _sz, _vp]
_lib.ks_scan.restype = _i
_lib.ks_scan_seeded.argtypes = [_i, _i, _i, _vp, _vp, _sz, _vp, _vp]
_lib.ks_scan_seeded.restype = _i
_lib.ks_scan_static.argtypes = [_i, _i, _i, _vp, _vp, _sz, _vp]
_lib.ks_scan_static.restype = _i
_lib.ks_mapreduce.argtypes = [_i, _i, _i, _vp, _sz, _vp, _vp]
_lib.ks_mapreduce.restype = _i
_lib.ks_mapreduce_result_bytes.argtypes = [_i, _i, _i]
_lib.ks_mapreduce_result_bytes.restype = _sz
_lib.ks_scan_map.argtypes = [_i, _i, _i, _i, _vp, _vp, _sz, _vp]
_lib.ks_scan_map.restype = _i
_lib.ks_scan_strided.argtypes = [_i, _i, _i, _vp, _sz, _vp, _sz, _sz, _vp]
_lib.ks_scan_strided.restype = _i
_lib.ks_map_supported.argtypes = [_i, _i, _i]
_lib.ks_map_supported.restype = _i
_lib.ks_scan_temp_bytes.argtypes = [_i, _i, _i, _sz]
_lib.ks_scan_temp_bytes.restype = _sz
_lib.ks_scan_with_temp.argtypes = [_i, _i, _i, _i, _vp, _vp, _sz, _vp, _sz, _vp]
_lib.ks_scan_with_temp.restype = _i
_lib.ks_scan_check.argtypes = [_vp]
_lib.ks_scan_check.restype = _i
_lib.ks_release_scratch.argtypes = [_vp]
_lib.ks_release_scratch.restype = _i
_lib.ks_scan_pair.argtypes = [_vp, _i, _vp, _vp, _sz, _vp]
_lib.ks_scan_pair.restype = _i
_lib.ks_mapreduce_pair.argtypes = [_vp, _vp, _sz, _vp, _vp]
_lib.ks_mapreduce_pair.restype = _i
_lib.ks_pair_elem_bytes.argtypes = [_vp]
_lib.ks_pair_elem_bytes.restype = _sz
_lib.ks_pair_supported.argtypes = [_i, _i]
_lib.ks_pair_supported.restype = _i
_lib.ks_elem_bytes.argtypes = [_i]
_lib.ks_elem_bytes.restype = _sz
_lib.ks_set_option.argtypes = [ctypes.c_char_p, ctypes.c_longlong]
_lib.ks_set_option.restype = _i
_lib.ks_get_option.argtypes = [ctypes.c_char_p]
_lib.ks_get_option.restype = ctypes.c_longlong
_lib.ks_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.ks_copy.restype = _i
_lib.ks_status_string.argtypes = [_i]
_lib.ks_status_string.restype = ctypes.c_char_p
_lib.ks_last_hip_error.argtypes = []
_lib.ks_last_hip_error.restype = _i
_lib.ks_version.argtypes = []
_lib.ks_version.restype = ctypes.c_char_p


class KsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.ks_status_string(status).decode()
        if status == KS_ERR_HIP:
            msg += f" [hip error {_lib.ks_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


def _check(status: int, where: str) -> None:
    if status != KS_OK:
        raise KsError(status, where)


# torch.cuda.current_stream() builds a Stream object (about 3 us, as much as the launch itself);
# the raw handle of the device's current stream comes straight from the C layer where torch has it.
_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream_ptr(stream, device_index=None) -> int:
    if stream is None:
        if _raw_current_stream is not None:
            return _raw_current_stream(torch.cuda.current_device() if device_index is None else device_index)
        stream = torch.cuda.current_stream(device_index)
    return int(stream.cuda_stream)


class _OnDeviceOf:
    """Make the tensor's device current for the call; free when it already is (the common case)."""

    def __init__(self, t: torch.Tensor):
        self._guard = None if t.device.index == torch.cuda.current_device() else torch.cuda.device(t.device)

    def __enter__(self):
        if self._guard is not None:
            self._guard.__enter__()

    def __exit__(self, *exc):
        if self._guard is not None:
            self._guard.__exit__(*exc)


_ELEM_BYTES: dict = {}
_RESULT_BYTES: dict = {}


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def _elements(t: torch.Tensor, dtype: str) -> int:
    if not t.is_cuda:
        raise ValueError("ks_scan works on device tensors only")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    eb = _ELEM_BYTES.get(dtype)
    if eb is None:   # asked of the library once per dtype: this runs on every call
        eb = _ELEM_BYTES[dtype] = int(_lib.ks_elem_bytes(DTYPES[dtype]))
    if _nbytes(t) % eb:
        raise ValueError(f"tensor of {_nbytes(t)} bytes is not a whole number of {dtype} elements")
    return _nbytes(t) // eb


def ks_scan(inp: torch.Tensor, out: torch.Tensor, *, dtype: str, op: str, inclusive: bool = True,
            stream=None) -> torch.Tensor:
    """out = scan(inp) with the library-owned workspace.  Asynchronous on the stream."""
    n = _elements(inp, dtype)
    if _elements(out, dtype) != n:
        raise ValueError("inp and out differ in size")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan(DTYPES[dtype], OPS[op], int(bool(inclusive)), inp.data_ptr(), out.data_ptr(), n,
                            _stream_ptr(stream, inp.device.index)), "ks_scan")
    return out


def ks_mapreduce(inp: torch.Tensor, out: torch.Tensor, *, dtype: str, op: str, map: str = "identity",
                 stream=None) -> torch.Tensor:
    """out[0] = op(map(inp[0]), ..., map(inp[n-1])), one launch; `out` holds one element of the result
    type (`dtype`, or what the map turns it into: see ks_mapreduce_result_bytes).  Asynchronous on the stream."""
    n = _elements(inp, dtype)
    if not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must be a contiguous device tensor")
    want = _RESULT_BYTES.get((dtype, map, op))
    if want is None:     # asked of the library once per triple
        want = _RESULT_BYTES[(dtype, map, op)] = ks_mapreduce_result_bytes(dtype=dtype, map=map, op=op)
    if want and _nbytes(out) != want:    # a triple the library does not take is for the library to refuse
        raise ValueError("out must hold exactly one element of the result type")
    with _OnDeviceOf(inp):
        _check(_lib.ks_mapreduce(DTYPES[dtype], MAPS[map], OPS[op], inp.data_ptr() if n else None, n, out.data_ptr(),
                                 _stream_ptr(stream, inp.device.index)), "ks_mapreduce")
    return out


def ks_mapreduce_result_bytes(*, dtype: str, op: str, map: str = "identity") -> int:
    """Size of what ks_mapreduce writes for this triple; 0 if it does not accept it."""
    return int(_lib.ks_mapreduce_result_bytes(DTYPES[dtype], MAPS[map], OPS[op]))


def ks_scan_seeded(inp: torch.Tensor, out: torch.Tensor, seed: torch.Tensor, *, dtype: str, op: str,
                   inclusive: bool = True, stream=None) -> torch.Tensor:
    """out[i] = seed op inp[0] op ... op inp[i]: one piece of a longer sequence; `seed` is a device tensor
    of one element (for instance a slice of the previous piece's output).  Asynchronous on the stream."""
    n = _elements(inp, dtype)
    if _elements(out, dtype) != n:
        raise ValueError("inp and out differ in size")
    if not seed.is_cuda or _nbytes(seed) != _ELEM_BYTES[dtype]:
        raise ValueError("seed must be a device tensor of exactly one element")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_seeded(DTYPES[dtype], OPS[op], int(bool(inclusive)), inp.data_ptr(), out.data_ptr(), n,
                                   seed.data_ptr(), _stream_ptr(stream, inp.device.index)), "ks_scan_seeded")
    return out


STATIC_SCRATCH_BYTES = 8 << 20


def ks_scan_static(inp: torch.Tensor, out: torch.Tensor, *, dtype: str, op: str, inclusive: bool = True,
                   stream=None) -> torch.Tensor:
    """out = scan(inp) using the library's static device scratch: allocates nothing; see ks_scan.h for the limit."""
    n = _elements(inp, dtype)
    if _elements(out, dtype) != n:
        raise ValueError("inp and out differ in size")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_static(DTYPES[dtype], OPS[op], int(bool(inclusive)), inp.data_ptr(), out.data_ptr(), n,
                                   _stream_ptr(stream, inp.device.index)), "ks_scan_static")
    return out


def ks_scan_map(inp: torch.Tensor, out: torch.Tensor, *, dtype: str, map: str, op: str, inclusive: bool = True,
                stream=None) -> torch.Tensor:
    """out = scan(op, map(inp)): the map-fused scan, library-owned workspace.  Asynchronous on the stream."""
    n = _elements(inp, dtype)
    if _elements(out, dtype) != n:
        raise ValueError("inp and out differ in size")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_map(DTYPES[dtype], MAPS[map], OPS[op], int(bool(inclusive)), inp.data_ptr(),
                                out.data_ptr(), n, _stream_ptr(stream, inp.device.index)), "ks_scan_map")
    return out


def ks_scan_strided(inp: torch.Tensor, out: torch.Tensor, *, dtype: str, op: str, n: int, in_stride: int = 1,
                    out_stride: int = 1, inclusive: bool = True, stream=None) -> torch.Tensor:
    """Scan of the strided views inp[::in_stride][:n] -> out[::out_stride][:n] of two contiguous device buffers
    (strides in elements of `dtype`)."""
    for t, stride in ((inp, in_stride), (out, out_stride)):
        if n > 0 and _elements(t, dtype) < (n - 1) * stride + 1:
            raise ValueError("tensor too small for the requested view")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_strided(DTYPES[dtype], OPS[op], int(bool(inclusive)), inp.data_ptr(), in_stride,
                                    out.data_ptr(), out_stride, n, _stream_ptr(stream, inp.device.index)),
               "ks_scan_strided")
    return out


def ks_map_supported(dtype: str, map: str, op: str) -> bool:
    return bool(_lib.ks_map_supported(DTYPES[dtype], MAPS[map], OPS[op]))


def ks_scan_temp_bytes(*, dtype: str, op: str, n: int, algo: str = "auto") -> int:
    return int(_lib.ks_scan_temp_bytes(DTYPES[dtype], OPS[op], ALGOS[algo], n))


def ks_scan_with_temp(inp: torch.Tensor, out: torch.Tensor, temp: torch.Tensor, *, dtype: str, op: str,
                      inclusive: bool = True, algo: str = "auto", stream=None) -> torch.Tensor:
    """out = scan(inp) using caller-owned device scratch `temp` (any dtype, 256-byte aligned)."""
    n = _elements(inp, dtype)
    if _elements(out, dtype) != n:
        raise ValueError("inp and out differ in size")
    if not temp.is_cuda or not temp.is_contiguous():
        raise ValueError("temp must be a contiguous device tensor")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_with_temp(DTYPES[dtype], OPS[op], int(bool(inclusive)), ALGOS[algo], inp.data_ptr(),
                                      out.data_ptr(), n, temp.data_ptr(), _nbytes(temp),
                                      _stream_ptr(stream, inp.device.index)),
               "ks_scan_with_temp")
    return out


def ks_scan_check(stream=None) -> None:
    """Synchronise the stream; raise KsError(KS_ERR_TIMEOUT) if a look-back wait was abandoned."""
    _check(_lib.ks_scan_check(_stream_ptr(stream)), "ks_scan_check")


def ks_pair_supported(dtype: str, op: str) -> bool:
    return bool(_lib.ks_pair_supported(DTYPES[dtype], OPS[op]))


def ks_elem_bytes(dtype: str) -> int:
    return int(_lib.ks_elem_bytes(DTYPES[dtype]))


def ks_set_option(name: str, value: int) -> None:
    _check(_lib.ks_set_option(name.encode(), int(value)), f"ks_set_option({name})")


def ks_get_option(name: str) -> int:
    return int(_lib.ks_get_option(name.encode()))


def ks_pair_elem_bytes(pair: int) -> int:
    """sizeof the element type of a pair compiled outside the library; 0 if `pair` is not one."""
    return int(_lib.ks_pair_elem_bytes(pair))


def _pair_elements(t: torch.Tensor, pair: int) -> int:
    eb = ks_pair_elem_bytes(pair)
    if eb == 0:
        raise ValueError("not a pair of this version of the library")
    if not t.is_cuda or not t.is_contiguous() or _nbytes(t) % eb:
        raise ValueError("tensor must be a contiguous device tensor of whole elements")
    return _nbytes(t) // eb


def ks_scan_pair(pair: int, inp: torch.Tensor, out: torch.Tensor, *, inclusive: bool = True, stream=None) -> torch.Tensor:
    """out = scan(inp) for a type and operator compiled outside the library: `pair` is the address that
    ks::Pair<T, Op>::entry() returned there (see include/ks_scan.h and examples/user_pair.hip)."""
    n = _pair_elements(inp, pair)
    if _pair_elements(out, pair) != n:
        raise ValueError("inp and out differ in size")
    with _OnDeviceOf(inp):
        _check(_lib.ks_scan_pair(pair, int(bool(inclusive)), inp.data_ptr(), out.data_ptr(), n,
                                 _stream_ptr(stream, inp.device.index)), "ks_scan_pair")
    return out


def ks_mapreduce_pair(pair: int, inp: torch.Tensor, out: torch.Tensor, *, stream=None) -> torch.Tensor:
    """out[0] = the left fold of inp for a pair compiled outside the library; `out` holds one element."""
    n = _pair_elements(inp, pair)
    if _pair_elements(out, pair) != 1:
        raise ValueError("out must hold exactly one element")
    with _OnDeviceOf(inp):
        _check(_lib.ks_mapreduce_pair(pair, inp.data_ptr() if n else None, n, out.data_ptr(),
                                      _stream_ptr(stream, inp.device.index)), "ks_mapreduce_pair")
    return out


def ks_release_scratch(stream=None) -> None:
    """Synchronise the stream and free the scratch the library caches for it (kept if a graph recorded it)."""
    _check(_lib.ks_release_scratch(_stream_ptr(stream)), "ks_release_scratch")


def ks_copy(inp: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
    """Vectorised device copy used as the bandwidth ceiling in measurements."""
    if _nbytes(inp) != _nbytes(out):
        raise ValueError("inp and out differ in size")
    _check(_lib.ks_copy(inp.data_ptr(), out.data_ptr(), _nbytes(inp), _stream_ptr(stream, inp.device.index)), "ks_copy")
    return out


def ks_version() -> str:
    return _lib.ks_version().decode()


def raw_library() -> ctypes.CDLL:
    """The ctypes handle, for tests that exercise argument validation with raw pointers."""
    return _lib


def ks_status_string(status: int) -> str:
    return _lib.ks_status_string(int(status)).decode()


def ks_last_hip_error() -> int:
    return int(_lib.ks_last_hip_error())
