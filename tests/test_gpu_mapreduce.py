"""GPU parity of ks_mapreduce (paper Sec. II-C / V-A) against the oracle's sequential left fold, through
the C ABI.  Integer and struct results bit for bit; float results within max(1e-4 |ref|, 1e-3) of the
oracle's float64 fold (min / max of floats exactly)."""
import sys

import numpy as np
import pytest
import torch

import ks_inputs
import oracle
from parity import FLOAT_TOL, KINDS, float_bound, random_input, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def reduce_on_gpu(ks, dtype, op, x, map_name="identity", d_in=None):
    d_in = to_device(x) if d_in is None else d_in
    one = to_device(x[:1]) if len(x) else to_device(np.zeros((1,) + x.shape[1:], x.dtype))
    out = torch.full_like(one, 0x55)
    ks.ks_mapreduce(d_in, out, dtype=dtype, op=op, map=map_name)
    ks.ks_scan_check()
    return to_host(out, x.dtype)[0]


def check(dtype, op, got, ref, what):
    if (dtype, op) in FLOAT_TOL:
        g, r = np.asarray(got, dtype=np.float64).reshape(-1), np.asarray(ref, dtype=np.float64).reshape(-1)
        assert np.all(np.abs(g - r) <= float_bound(r)), f"{what}: gpu={g} ref={r}"
    elif np.asarray(got).dtype.names:
        assert got == ref, f"{what}: gpu={got} ref={ref}"
    else:
        assert np.array_equal(np.asarray(got), np.asarray(ref).astype(np.asarray(got).dtype)), f"{what}: gpu={got} ref={ref}"


def run_elems(ks, dtype):
    eb = ks.ks_elem_bytes(dtype)
    rows = 9 if (8 * 16) % eb else 8                       # a lane's rows * 16 bytes hold whole elements
    return 64 * rows * 16 // eb                            # elements one wave folds per step (at most)


@pytest.mark.parametrize("dtype,op", sorted(KINDS))
def test_every_pair_edge_sizes(ks, dtype, op):
    oop, odt, _, _ = KINDS[(dtype, op)]
    run = run_elems(ks, dtype)
    sizes = [0, 1, 2, 63, 64, 65, run - 1, run, run + 1, 4 * run - 1, 4 * run, 4 * run + 1, 37 * run + 5,
             2048 * 4 * run - 1, 2048 * 4 * run + 1, 3 * 2048 * 4 * run + 12345]
    for n in sizes:
        x = random_input(dtype, op, n, seed=500 + n % 89)
        say(f"[case] mapreduce ({dtype},{op}) n={n}")
        check(dtype, op, reduce_on_gpu(ks, dtype, op, x), oracle.mapreduce("identity", oop, odt, x), f"({dtype},{op}) n={n}")


MAP_TRIPLES = [("f32", "square", "sum"), ("f32", "abs", "sum"), ("f32", "abs", "max"), ("f64", "square", "sum"),
               ("i32", "nonzero", "sum"), ("i32", "abs", "max"), ("i32", "square", "sum"), ("u64", "nonzero", "sum")]


@pytest.mark.parametrize("dtype,map_name,op", MAP_TRIPLES)
def test_mapped_triples(ks, dtype, map_name, op):
    oop, odt, npdt, _ = KINDS[(dtype, op)]
    rng = np.random.default_rng(77)
    for n in (1, 5, 1000, 70_001, 5_000_003):
        if np.issubdtype(npdt, np.integer):
            x = (rng.integers(0, 3, size=n) * rng.integers(-1000, 1000, size=n)).astype(npdt)   # one third zeros
        else:
            x = rng.uniform(-2.0, 2.0, size=n).astype(npdt)
        say(f"[case] mapreduce ({dtype},{map_name},{op}) n={n}")
        got = reduce_on_gpu(ks, dtype, op, x, map_name)
        ref = oracle.mapreduce(map_name, oop, odt, x)
        check(dtype, op, got, ref, f"({dtype},{map_name},{op}) n={n}")
    assert ks.ks_map_supported(dtype, map_name, op)
    with pytest.raises(ks.KsError) as e:
        ks.ks_mapreduce(torch.zeros(4, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"),
                        dtype="i32", op="min", map="square")
    assert e.value.status == ks.KS_ERR_UNSUPPORTED


def test_closed_forms_and_operand_order(ks):
    n = (1 << 24) + 12345
    say("[case] mapreduce closed forms")
    assert int(reduce_on_gpu(ks, "i32", "sum", np.ones(n, np.int32))) == n
    i = np.arange(n, dtype=np.uint64)
    assert int(reduce_on_gpu(ks, "u64", "sum", i)) == n * (n - 1) // 2
    # double accumulation: exact past 2^24, rounded to float32 once at the end
    assert float(reduce_on_gpu(ks, "f32", "sum", np.ones(n, np.float32))) == float(np.float32(n))
    # Fibonacci matrices: the ordered product of n copies of [[1,1],[1,0]]
    m = 70 * 1024 + 5
    x = np.tile(np.array([[1, 1, 1, 0]], dtype=np.uint32), (m, 1))
    a, b, mask = 1, 0, (1 << 32) - 1
    for _ in range(m):
        a, b = (a + b) & mask, a
    assert reduce_on_gpu(ks, "mat2_u32", "mat2_mul", x).tolist() == [a, b, b, (a - b) & mask]
    # alternating non-commuting factors: order kept across lanes, runs, waves and workgroups
    y = np.where((np.arange(3_000_001) % 2 == 0)[:, None], np.array([[1, 1, 0, 1]]), np.array([[1, 0, 1, 1]])).astype(np.uint32)
    assert reduce_on_gpu(ks, "mat2_u32", "mat2_mul", y).tolist() == oracle.mapreduce("identity", "mat2", "u32", y).tolist()


def test_back_to_back_with_scans_on_the_same_stream(ks):
    # the reduction shares the stream's scratch and epoch counter with ks_scan: interleave them,
    # sizes going up and down; `out` inside the input is allowed
    rng = np.random.default_rng(5)
    for it in range(12):
        n = int(rng.integers(1, 6_000_000))
        x = rng.integers(-1000, 1000, size=n).astype(np.int32)
        d = to_device(x)
        scanned = torch.empty_like(d)
        ks.ks_scan(d, scanned, dtype="i32", op="sum")
        total = torch.zeros(1, dtype=torch.int32, device="cuda")
        ks.ks_mapreduce(d, total, dtype="i32", op="sum")
        ks.ks_mapreduce(d, d[:1], dtype="i32", op="max")          # result over the first input element
        ks.ks_scan_check()
        say(f"[case] scan + mapreduce interleaved, n={n}")
        assert int(total[0]) == int(scanned[-1]) == int(np.sum(x, dtype=np.int32))
        assert int(d[0]) == int(x.max())


def test_full_size_configs(ks):
    for name, n in (("f32_sum", 1 << 28), ("argmax", 1 << 26), ("affine", 1 << 26)):
        w = ks_inputs.WORKLOADS[name]
        oop, odt, _, _ = KINDS[(w.dtype, w.op)]
        parts = [to_device(c) for c in ks_inputs.chunks(name, n)]
        d_in = torch.cat(parts)
        del parts
        out = torch.empty_like(d_in[:1])
        say(f"[case] mapreduce workload={name} n={n}")
        ks.ks_mapreduce(d_in, out, dtype=w.dtype, op=w.op)
        ks.ks_scan_check()
        stream = oracle.ScanStream(oop, odt, True)
        last = None
        for c in ks_inputs.chunks(name, n):
            last = stream.feed(c)[-1]
        got = to_host(out, next(iter(ks_inputs.chunks(name, 1))).dtype)[0]
        check(w.dtype, w.op, got, last, name)
        del d_in


# ---- bytes: the 8-bit types of the paper's mapreduce benchmark (Sec. VII-B, Tables I and III) ----
BYTE_MAPS = {"unit_float8": np.float32, "widen64": np.uint64, "identity": np.uint8}


def reduce_bytes_on_gpu(ks, d_in, map_name):
    """d_in: a uint8 device tensor (any slice); returns the result as a numpy scalar of the result type."""
    rt = BYTE_MAPS[map_name]
    out = torch.full((np.dtype(rt).itemsize,), 0x55, dtype=torch.uint8, device="cuda")
    ks.ks_mapreduce(d_in, out, dtype="u8", op="sum", map=map_name)
    ks.ks_scan_check()
    return out.cpu().numpy().view(rt)[0]


def check_bytes(map_name, got, x, what):
    ref = oracle.mapreduce(map_name, "sum", "u8", x)
    if map_name == "unit_float8":
        assert abs(float(got) - float(ref)) <= float_bound(np.array([float(ref)]))[0], f"{what}: gpu={got} ref={ref}"
    else:
        assert int(got) == int(ref), f"{what}: gpu={got} ref={ref}"


def test_unit_float8_levels_one_by_one(ks):
    # n = 1: the result is the level itself, promoted to float32: bit for bit the oracle's, for all 256 codes
    codes = to_device(np.arange(256, dtype=np.uint8))
    levels = oracle.apply_map("unit_float8", np.arange(256, dtype=np.uint8))
    say("[case] mapreduce unit_float8: the 256 levels")
    for c in range(256):
        got = reduce_bytes_on_gpu(ks, codes[c:c + 1], "unit_float8")
        assert got.dtype == np.float32 and got == levels[c], (c, got, levels[c])


@pytest.mark.parametrize("map_name", sorted(BYTE_MAPS))
def test_byte_sums_edge_sizes_and_offsets(ks, map_name):
    run = 64 * 4 * 16                       # bytes one wave folds per step
    sizes = [0, 1, 2, 3, 4, 5, 15, 16, 17, 63, 64, 65, 1023, 1024, 1025, run - 1, run, run + 1, 4 * run - 3, 4 * run,
             4 * run + 1, 37 * run + 5, 512 * 4 * run - 1, 512 * 4 * run + 2, 3 * 512 * 4 * run + 12345]
    x_all = ks_inputs.random_codes(sizes[-1] + 16, seed=31)
    d_all = to_device(x_all)
    for n in sizes:
        for off in ((0, 1, 2, 3, 5) if n < 70_000 else (0, 3)):      # the input need not start on a dword
            say(f"[case] mapreduce (u8,{map_name},sum) n={n} +{off}")
            got = reduce_bytes_on_gpu(ks, d_all[off:off + n], map_name)
            check_bytes(map_name, got, x_all[off:off + n], f"(u8,{map_name}) n={n} +{off}")


def test_byte_sums_closed_forms(ks):
    n = (1 << 25) + 77
    full = torch.full((n,), 255, dtype=torch.uint8, device="cuda")
    say(f"[case] mapreduce u8 closed forms n={n}")
    assert int(reduce_bytes_on_gpu(ks, full, "widen64")) == 255 * n          # > 2^32: carried in 64 bits
    assert int(reduce_bytes_on_gpu(ks, full, "identity")) == (255 * n) % 256
    assert float(reduce_bytes_on_gpu(ks, full, "unit_float8")) == float(np.float32(n))   # level 255 = +1
    full.fill_(0)
    assert float(reduce_bytes_on_gpu(ks, full, "unit_float8")) == -float(np.float32(n))  # level 0 = -1
    # every level equally often: the levels cancel in pairs and the exact sum is 0.  The input is as
    # regular as can be (every lane adds the same 16 levels in every run), so the float32 roundings
    # inside the runs repeat instead of averaging out; what bounds them is the error of a
    # recursive float32 sum of the 64 terms of one lane and run, 63 * 2^-24 * sum |level|
    # (above the run the sum is carried in double)
    reps = 1 << 14
    cyc = to_device(np.tile(np.arange(256, dtype=np.uint8), reps))
    sum_abs = reps * float(np.abs(oracle.apply_map("unit_float8", np.arange(256, dtype=np.uint8)).astype(np.float64)).sum())
    assert abs(float(reduce_bytes_on_gpu(ks, cyc, "unit_float8"))) <= 63 * 2.0 ** -24 * sum_abs
    assert abs(float(reduce_bytes_on_gpu(ks, cyc, "unit_float8"))) <= 1e-8 * sum_abs    # and far inside it
    # the scans refuse bytes, and so does every other operator
    with pytest.raises(ks.KsError) as e:
        ks.ks_scan(cyc, torch.empty_like(cyc), dtype="u8", op="sum")
    assert e.value.status == ks.KS_ERR_UNSUPPORTED
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="max") == 0


def test_byte_sums_at_the_paper_sizes(ks):
    # n = 10^6 ... 10^9 (Tables I and III); uniform codes (the sum of the levels wanders around zero)
    # and codes skewed upwards (it grows)
    for n, skew in ((10 ** 6, 0.0), (10 ** 7, 0.25), (10 ** 8, 0.0), (10 ** 9, 0.25)):
        x = ks_inputs.random_codes(n, seed=41, skew=skew)
        d = to_device(x)
        for map_name in sorted(BYTE_MAPS):
            say(f"[case] mapreduce (u8,{map_name},sum) n={n} skew={skew}")
            check_bytes(map_name, reduce_bytes_on_gpu(ks, d, map_name), x, f"(u8,{map_name}) n={n} skew={skew}")
        del d, x


# ---- 16-bit floats, reduced after promotion to float32 ----
@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_sixteen_bit_floats(ks, kind):
    run = 64 * 4 * 8                        # elements one wave folds per step
    sizes = [0, 1, 2, 3, 7, 8, 9, 63, 64, 65, run - 1, run, run + 1, 4 * run + 3, 37 * run + 5, 512 * 4 * run + 1,
             3 * 512 * 4 * run + 12345, (1 << 27) + 3]
    x_all = ks_inputs.random_half_bits(kind, sizes[-1] + 8, seed=51)
    d_all = torch.from_numpy(x_all.view(np.int16)).cuda()
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    for n in sizes:
        for off in ((0, 1, 2, 3) if n < 100_000 else (0, 1)):     # the input need not start on a dword
            x = x_all[off:off + n]
            for op in ("sum", "max", "min"):
                say(f"[case] mapreduce ({kind},widen_f32,{op}) n={n} +{off}")
                out.fill_(123.0)
                ks.ks_mapreduce(d_all[off:off + n], out, dtype=kind, op=op, map="widen_f32")
                ks.ks_scan_check()
                got, ref = float(out.cpu()[0]), float(oracle.mapreduce("widen_f32", op, kind, x))
                if op == "sum":
                    assert abs(got - ref) <= float_bound(np.array([ref]))[0], (kind, op, n, off, got, ref)
                else:
                    assert got == ref, (kind, op, n, off, got, ref)
    # n ones: exact as long as the count is a float32
    one = {"bf16": 0x3F80, "f16": 0x3C00}[kind]
    ones = torch.full((1 << 24,), one, dtype=torch.int16, device="cuda")
    ks.ks_mapreduce(ones, out, dtype=kind, op="sum", map="widen_f32")
    ks.ks_scan_check()
    assert float(out.cpu()[0]) == float(1 << 24)
    with pytest.raises(ks.KsError) as e:
        ks.ks_mapreduce(ones, torch.empty(2, dtype=torch.uint8, device="cuda"), dtype=kind, op="sum")
    assert e.value.status == ks.KS_ERR_UNSUPPORTED      # no reduction in the 16-bit type itself


def test_recorded_into_a_graph(ks):
    n = 3_000_001
    xs = [np.random.default_rng(90 + r).integers(-50, 50, size=n).astype(np.int32) for r in range(3)]
    d_in = to_device(xs[0])
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ks.ks_mapreduce(d_in, out, dtype="i32", op="sum")     # eager first: allocates the stream's scratch
    ks.ks_scan_check(s)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        ks.ks_mapreduce(d_in, out, dtype="i32", op="sum")
    for r in range(3):
        d_in.copy_(to_device(xs[r]))
        out.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            graph.replay()
            graph.replay()
        ks.ks_scan_check(s)
        say(f"[case] mapreduce graph replay {r}")
        assert int(out[0]) == int(np.sum(xs[r], dtype=np.int32))
