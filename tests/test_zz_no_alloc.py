"""ks_scan_static, the entry point that allocates nothing (static device scratch), against
ks_scan_with_temp on the same inputs, through the C ABI.  Integer and struct results must agree
bit for bit; float32 sums within the float bar of tests/parity.py (the two calls may group tile
aggregates differently in the last bits)."""
import ctypes

import numpy as np
import pytest
import torch

from parity import assert_matches, random_input, reference, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


def _with_temp(ks, dtype, op, d_in, n, inclusive):
    out = torch.empty_like(d_in)
    temp = torch.empty(ks.ks_scan_temp_bytes(dtype=dtype, op=op, n=n), dtype=torch.uint8, device="cuda")
    ks.ks_scan_with_temp(d_in, out, temp, dtype=dtype, op=op, inclusive=inclusive)
    return out


@pytest.mark.parametrize("dtype,op,sizes", [
    ("i32", "sum", (40_000_003, 1_000_001, 77)),                     # several rounds, then smaller, then one tile
    ("f32", "sum", (30_000_017, 2_500_000)),
    ("u64", "sum", (9_000_001, 300_007)),
    ("argmax_i32_cnt64", "argmax_count", (5_000_011, 5_000_010, 70_001)),
    ("mat2_u32", "mat2_mul", (3_000_001, 65)),
])
def test_static_scratch_matches_caller_scratch_on_calls_in_a_row(ks, dtype, op, sizes):
    lib = ks.raw_library()
    stream = torch.cuda.current_stream().cuda_stream
    for inclusive in (True, False):
        for n in sizes:                                    # same array on every call: each one smaller than the last
            x = random_input(dtype, op, n, seed=n % 7919)
            d_in = to_device(x)
            d_out = torch.empty_like(d_in)
            print(f"[case] ks_scan_static ({dtype},{op}) n={n} inclusive={inclusive}", flush=True)
            st = lib.ks_scan_static(ks.DTYPES[dtype], ks.OPS[op], int(inclusive), d_in.data_ptr(), d_out.data_ptr(), n,
                                    stream)
            assert st == ks.KS_OK, ks.ks_status_string(st)
            ks.ks_scan_check()
            want = _with_temp(ks, dtype, op, d_in, n, inclusive)
            ks.ks_scan_check()
            if dtype == "f32":
                ref = reference(dtype, op, x, inclusive)
                assert_matches(dtype, op, to_host(d_out, x.dtype), ref, "static")
                assert_matches(dtype, op, to_host(want, x.dtype), ref, "with_temp")
                assert torch.allclose(d_out, want, rtol=1e-4, atol=1e-3)
            else:
                assert torch.equal(d_out, want), (dtype, op, n, inclusive)
                assert_matches(dtype, op, to_host(d_out, x.dtype), reference(dtype, op, x, inclusive), "static")


def test_static_scratch_refuses_what_does_not_fit_and_allocates_nothing(ks):
    lib = ks.raw_library()
    stream = torch.cuda.current_stream().cuda_stream
    # beyond the stated maximum: refused with a clear error, nothing launched, the output untouched
    n = 1 << 27
    assert ks.ks_scan_temp_bytes(dtype="argmax_i32_cnt64", op="argmax_count", n=n) > ks.STATIC_SCRATCH_BYTES
    d_in = torch.zeros((n, 4), dtype=torch.int32, device="cuda")
    d_out = torch.full_like(d_in, 7)
    st = lib.ks_scan_static(ks.DTYPES["argmax_i32_cnt64"], ks.OPS["argmax_count"], 1, d_in.data_ptr(), d_out.data_ptr(), n,
                            stream)
    assert st == ks.KS_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((d_out[:1000] == 7).all()) and bool((d_out[-1000:] == 7).all())
    del d_in, d_out
    # the largest float32 input that fits; device memory in use must not move across the calls
    n = 1 << 29
    assert ks.ks_scan_temp_bytes(dtype="f32", op="sum", n=n) <= ks.STATIC_SCRATCH_BYTES
    x = torch.ones(n, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        st = lib.ks_scan_static(ks.DTYPES["f32"], ks.OPS["sum"], 1, x.data_ptr(), y.data_ptr(), n, stream)
        assert st == ks.KS_OK
    ks.ks_scan_check()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before, (free_before, free_after)
    assert float(y[(1 << 24) - 1]) == float(1 << 24)          # all-ones: exact up to 2^24
    assert abs(float(y[-1]) - n) <= 1e-4 * n
    # argument checks are those of ks_scan
    assert lib.ks_scan_static(99, 0, 1, x.data_ptr(), y.data_ptr(), 16, stream) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan_static(ks.DTYPES["f32"], ks.OPS["sum"], 1, x.data_ptr(), x.data_ptr() + 4, 16, stream) == ks.KS_ERR_OVERLAP
    assert lib.ks_scan_static(ks.DTYPES["f32"], ks.OPS["sum"], 1, 0, 0, 0, stream) == ks.KS_OK


def test_static_scratch_call_recorded_into_a_graph(ks):
    # nothing to allocate and no scratch to prepare: recorded on a fresh stream, replayed with new inputs
    # (one eager call first: the first launch of a kernel loads its code, which must not happen under capture)
    dtype, op, n = "i32", "sum", 5_000_003
    xs = [random_input(dtype, op, n, seed=80 + r) for r in range(3)]
    d_in = to_device(xs[0])
    d_out = torch.empty_like(d_in)
    ks.ks_scan_static(d_in, d_out, dtype=dtype, op=op)
    ks.ks_scan_check()
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        ks.ks_scan_static(d_in, d_out, dtype=dtype, op=op, stream=s)
    for r in range(3):
        d_in.copy_(to_device(xs[r]))
        d_out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ks.ks_scan_check(s)
        assert np.array_equal(to_host(d_out, xs[r].dtype), reference(dtype, op, xs[r], True)), r
