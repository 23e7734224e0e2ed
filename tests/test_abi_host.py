"""CPU-only checks of the C-ABI boundary: the library loads, exports every declared symbol, and its
host-side validation answers without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ks_scan.h")


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ks_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ["ks_scan", "ks_scan_temp_bytes", "ks_scan_with_temp", "ks_scan_check", "ks_copy",
                 "ks_status_string", "ks_last_hip_error", "ks_version"]:
        assert must in names


def test_library_exports_every_declared_symbol(ks):
    lib = ctypes.CDLL(ks.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert sorted(ks.EXPORTS) == declared_functions()


def test_python_binding_has_the_same_names(ks):
    for name in declared_functions():
        assert hasattr(ks, name), name


def test_binding_enums_match_the_header(ks):
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    consts = {name: int(value) for name, value in re.findall(r"\b(KS_[A-Z0-9_]+)\s*=\s*(-?\d+)", text)}
    for table, prefix in ((ks.DTYPES, "KS_"), (ks.OPS, "KS_"), (ks.MAPS, "KS_MAP_"), (ks.ALGOS, "KS_ALGO_")):
        for name, value in table.items():
            assert consts[prefix + name.upper()] == value, (prefix, name)
    assert len(ks.DTYPES) == consts["KS_DTYPE_COUNT"] and len(ks.OPS) == consts["KS_OP_COUNT"]
    assert len(ks.MAPS) == consts["KS_MAP_COUNT"]
    for name, value in consts.items():
        if name.startswith("KS_ERR_") or name == "KS_OK":
            assert getattr(ks, name) == value, name
    # every element type has a size, and the binding's scratch limit is the header's
    for name in ks.DTYPES:
        assert ks.ks_elem_bytes(name) in (1, 2, 4, 8, 12, 16, 32), name
    m = re.search(r"#define\s+KS_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert ks.STATIC_SCRATCH_BYTES == int(m.group(1)) << int(m.group(2))


def test_enums_and_sizes(ks):
    assert ks.ks_elem_bytes("f32") == 4 and ks.ks_elem_bytes("u64") == 8
    assert ks.ks_elem_bytes("affine_f32") == 8 and ks.ks_elem_bytes("argmax_i32_cnt64") == 16
    lib = ks.raw_library()
    assert lib.ks_elem_bytes(99) == 0
    for dt in ["i32", "u32", "i64", "u64", "f32", "f64"]:
        for op in ["sum", "min", "max"]:
            assert ks.ks_pair_supported(dt, op)
    assert ks.ks_pair_supported("affine_f32", "affine_compose")
    assert ks.ks_pair_supported("argmax_i32_cnt64", "argmax_count")
    assert ks.ks_pair_supported("mat2_u32", "mat2_mul") and ks.ks_pair_supported("quat_f32", "quat_mul")
    assert not ks.ks_pair_supported("f32", "affine_compose")
    assert not ks.ks_pair_supported("affine_f32", "sum")
    # element sizes other than 4, 8 and 16 bytes
    assert ks.ks_elem_bytes("mat2_u64") == 32 and ks.ks_elem_bytes("range_i32_cnt32") == 12
    assert ks.ks_pair_supported("mat2_u64", "mat2_mul") and ks.ks_pair_supported("range_i32_cnt32", "range_count")
    assert not ks.ks_pair_supported("mat2_u64", "sum")
    for dt in ("mat2_u64", "range_i32_cnt32"):
        op = "mat2_mul" if dt == "mat2_u64" else "range_count"
        for n in (1, 1000, 10**6, 10**9):
            assert ks.ks_scan_temp_bytes(dtype=dt, op=op, n=n, algo="lookback") % 256 == 0
            assert ks.ks_scan_temp_bytes(dtype=dt, op=op, n=n, algo="reduce_then_scan") >= 256


def test_mapreduce_and_static_argument_checks_need_no_gpu(ks):
    lib = ks.raw_library()
    lib.ks_mapreduce.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.ks_mapreduce(99, 0, 0, None, 0, 16, None) == ks.KS_ERR_INVALID_ARG          # bad dtype
    assert lib.ks_mapreduce(0, 9, 0, None, 0, 16, None) == ks.KS_ERR_INVALID_ARG           # bad map
    assert lib.ks_mapreduce(4, 1, 1, None, 0, 16, None) == ks.KS_ERR_UNSUPPORTED           # (f32, square, min) is no triple
    assert lib.ks_mapreduce(4, 0, 0, None, 0, None, None) == ks.KS_ERR_INVALID_ARG         # no output
    assert lib.ks_mapreduce(4, 0, 0, None, 5, 16, None) == ks.KS_ERR_INVALID_ARG           # n > 0 without input
    assert lib.ks_mapreduce(4, 0, 0, 18, 5, 16, None) == ks.KS_ERR_MISALIGNED
    lib.ks_scan_static.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert lib.ks_scan_static(4, 0, 1, None, None, 0, None) == ks.KS_OK                    # n == 0: nothing to do
    assert lib.ks_scan_static(4, 0, 1, None, 16, 4, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan_static(4, 3, 1, 16, 32, 4, None) == ks.KS_ERR_UNSUPPORTED           # (f32, affine_compose)
    assert lib.ks_scan_static(7, 4, 1, 1 << 40, 1 << 41, 1 << 27, None) == ks.KS_ERR_WORKSPACE   # beyond the static scratch


def test_bytes_are_reduced_and_not_scanned(ks):
    # the 8-bit types of the paper's mapreduce benchmark (Sec. VII-B): three sums over uint8, no scan
    U8, SUM = ks.DTYPES["u8"], ks.OPS["sum"]
    assert ks.ks_elem_bytes("u8") == 1
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="sum", map="unit_float8") == 4      # a float
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="sum", map="widen64") == 8          # a uint64
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="sum", map="identity") == 1         # modulo 2^8
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="max") == 0
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="sum", map="square") == 0
    assert ks.ks_mapreduce_result_bytes(dtype="f32", op="sum", map="unit_float8") == 0     # the map takes bytes only
    assert ks.ks_mapreduce_result_bytes(dtype="f32", op="sum") == 4
    assert ks.ks_mapreduce_result_bytes(dtype="argmax_i32_cnt64", op="argmax_count") == 16
    assert ks.ks_mapreduce_result_bytes(dtype="i32", op="sum", map="nonzero") == 4
    assert ks.ks_mapreduce_result_bytes(dtype="mat2_u64", op="mat2_mul") == 32
    assert ks.ks_mapreduce_result_bytes(dtype="range_i32_cnt32", op="range_count") == 12
    # 16-bit floats: sum, minimum and maximum after promotion to float, nothing else
    for dt in ("bf16", "f16"):
        assert ks.ks_elem_bytes(dt) == 2
        assert all(ks.ks_pair_supported(dt, op) for op in ("sum", "min", "max"))      # scanned as well
        assert not ks.ks_pair_supported(dt, "affine_compose")
        for op in ("sum", "min", "max"):
            assert ks.ks_mapreduce_result_bytes(dtype=dt, op=op, map="widen_f32") == 4
        assert ks.ks_mapreduce_result_bytes(dtype=dt, op="sum") == 0
        assert ks.ks_mapreduce_result_bytes(dtype=dt, op="sum", map="unit_float8") == 0
    assert ks.ks_mapreduce_result_bytes(dtype="u8", op="sum", map="widen_f32") == 0
    lib16 = ks.raw_library()
    lib16.ks_scan.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    BF = ks.DTYPES["bf16"]
    assert lib16.ks_scan(BF, ks.OPS["sum"], 1, 0x10000002, 0x20000000, 16, None) == ks.KS_ERR_MISALIGNED   # scans: dwords
    assert lib16.ks_scan(BF, ks.OPS["sum"], 1, 0x10000000, 0x20000002, 16, None) == ks.KS_ERR_MISALIGNED
    assert ks.ks_scan_temp_bytes(dtype="bf16", op="sum", n=10 ** 6) >= 256
    lib = ks.raw_library()
    assert lib.ks_mapreduce_result_bytes(99, 0, 0) == 0 and lib.ks_mapreduce_result_bytes(U8, 99, SUM) == 0
    assert not ks.ks_pair_supported("u8", "sum") and not ks.ks_map_supported("u8", "unit_float8", "sum")
    assert ks.ks_scan_temp_bytes(dtype="u8", op="sum", n=1000) == 0
    lib.ks_scan.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert lib.ks_scan(U8, SUM, 1, 0x10000000, 0x20000000, 16, None) == ks.KS_ERR_UNSUPPORTED
    lib.ks_scan_strided.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t,
                                                         ctypes.c_size_t, ctypes.c_void_p]
    assert lib.ks_scan_strided(U8, SUM, 1, 0x10000000, 2, 0x20000000, 2, 16, None) == ks.KS_ERR_UNSUPPORTED
    lib.ks_mapreduce.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.ks_mapreduce(U8, ks.MAPS["square"], SUM, 0x10000000, 5, 0x20000000, None) == ks.KS_ERR_UNSUPPORTED
    assert lib.ks_mapreduce(U8, ks.MAPS["widen64"], ks.OPS["max"], 0x10000000, 5, 0x20000000, None) == ks.KS_ERR_UNSUPPORTED
    # the input may start at any byte; the result must be aligned to its own type
    assert lib.ks_mapreduce(U8, ks.MAPS["widen64"], SUM, 0x10000003, 5, 0x20000004, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_mapreduce(U8, ks.MAPS["unit_float8"], SUM, 0x10000003, 5, 0x20000002, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_mapreduce(U8, ks.MAPS["unit_float8"], SUM, None, 5, 0x20000000, None) == ks.KS_ERR_INVALID_ARG


def test_pairs_compiled_outside_the_library(ks):
    # the example of a caller's own types and operators is built with the library; its pairs are
    # recognised by their tag, anything else is refused before any GPU work
    import os
    user = ctypes.CDLL(os.path.join(os.path.dirname(ks.LIB_PATH), "examples", "libks_user_pair.so"))
    pairs = {}
    for name, size in (("affine_u32", 8), ("stats24", 24)):
        fn = getattr(user, f"ks_user_{name}_pair")
        fn.restype = ctypes.c_void_p
        pairs[name] = fn()
        assert ks.ks_pair_elem_bytes(pairs[name]) == size
    lib = ks.raw_library()
    junk = ctypes.create_string_buffer(256)
    assert ks.ks_pair_elem_bytes(ctypes.addressof(junk)) == 0 and ks.ks_pair_elem_bytes(None) == 0
    assert lib.ks_scan_pair(ctypes.addressof(junk), 1, 0x10000000, 0x20000000, 16, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_mapreduce_pair(None, 0x10000000, 16, 0x20000000, None) == ks.KS_ERR_INVALID_ARG
    good = pairs["stats24"]
    assert lib.ks_scan_pair(good, 1, None, None, 0, None) == ks.KS_OK                           # n == 0
    assert lib.ks_scan_pair(good, 1, None, 0x20000000, 16, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan_pair(good, 1, 0x10000004, 0x20000000, 16, None) == ks.KS_ERR_MISALIGNED  # 8-byte fields
    assert lib.ks_scan_pair(good, 1, 0x10000000, 0x10000018, 16, None) == ks.KS_ERR_OVERLAP
    assert lib.ks_mapreduce_pair(good, 0x10000000, 16, None, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_mapreduce_pair(good, 0x10000000, 16, 0x20000004, None) == ks.KS_ERR_MISALIGNED


def test_seeded_scan_argument_checks_need_no_gpu(ks):
    lib = ks.raw_library()
    I32, SUM = ks.DTYPES["i32"], ks.OPS["sum"]
    assert lib.ks_scan_seeded(I32, SUM, 1, None, None, 0, None, None) == ks.KS_OK                           # n == 0
    assert lib.ks_scan_seeded(I32, SUM, 1, 0x10000000, 0x20000000, 16, None, None) == ks.KS_ERR_INVALID_ARG  # no seed
    assert lib.ks_scan_seeded(I32, SUM, 1, 0x10000000, 0x20000000, 16, 0x30000002, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan_seeded(I32, SUM, 1, 0x10000002, 0x20000000, 16, 0x30000000, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan_seeded(I32, SUM, 1, 0x10000000, 0x10000008, 16, 0x30000000, None) == ks.KS_ERR_OVERLAP
    assert lib.ks_scan_seeded(ks.DTYPES["u8"], SUM, 1, 0x10000000, 0x20000000, 16, 0x30000000, None) == ks.KS_ERR_UNSUPPORTED
    assert lib.ks_scan_seeded(99, SUM, 1, 0x10000000, 0x20000000, 16, 0x30000000, None) == ks.KS_ERR_INVALID_ARG
    # 16-bit floats: the arrays on dwords, the seed at any element
    BF = ks.DTYPES["bf16"]
    assert lib.ks_scan_seeded(BF, SUM, 1, 0x10000000, 0x20000000, 16, 0x30000001, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan_seeded(BF, SUM, 1, 0x10000002, 0x20000000, 16, 0x30000002, None) == ks.KS_ERR_MISALIGNED


def test_map_triples(ks):
    for triple in [("f32", "square", "sum"), ("f32", "abs", "sum"), ("f32", "abs", "max"), ("f64", "square", "sum"),
                   ("i32", "nonzero", "sum"), ("i32", "abs", "max"), ("i32", "square", "sum"), ("u64", "nonzero", "sum")]:
        assert ks.ks_map_supported(*triple), triple
    assert ks.ks_map_supported("u64", "identity", "sum")          # identity = the plain pair
    assert not ks.ks_map_supported("affine_f32", "square", "affine_compose")
    assert not ks.ks_map_supported("f32", "nonzero", "min")
    lib = ks.raw_library()
    # an unknown triple is refused before any GPU work; n == 0 of a known one is a no-op
    assert lib.ks_scan_map(ks.DTYPES["f32"], ks.MAPS["nonzero"], ks.OPS["min"], 1, 0x10000000, 0x20000000, 16, None) \
        == ks.KS_ERR_UNSUPPORTED
    assert lib.ks_scan_map(ks.DTYPES["f32"], ks.MAPS["square"], ks.OPS["sum"], 1, None, None, 0, None) == ks.KS_OK
    assert lib.ks_scan_map(ks.DTYPES["f32"], ks.MAPS["square"], ks.OPS["sum"], 1, None, 0x20000000, 16, None) \
        == ks.KS_ERR_INVALID_ARG


def test_strided_validation(ks):
    lib = ks.raw_library()
    f32, su = ks.DTYPES["f32"], ks.OPS["sum"]
    A, B = 0x10000000, 0x20000000
    assert lib.ks_scan_strided(f32, su, 1, A, 3, B, 2, 0, None) == ks.KS_OK                     # n == 0: nothing to do
    assert lib.ks_scan_strided(f32, su, 1, A, 0, B, 2, 16, None) == ks.KS_ERR_INVALID_ARG       # zero stride
    assert lib.ks_scan_strided(f32, su, 1, A, 1 << 21, B, 2, 16, None) == ks.KS_ERR_INVALID_ARG   # stride limit
    assert lib.ks_scan_strided(f32, su, 1, None, 3, B, 2, 16, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan_strided(f32, su, 1, A + 2, 3, B, 2, 16, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan_strided(f32, su, 1, A, 3, A + 4, 3, 16, None) == ks.KS_ERR_OVERLAP       # interleaved columns
    assert lib.ks_scan_strided(f32, su, 1, A, 3, A, 2, 16, None) == ks.KS_ERR_OVERLAP           # same base, other stride
    assert lib.ks_scan_strided(ks.DTYPES["f32"], ks.OPS["affine_compose"], 1, A, 3, B, 2, 16, None) == ks.KS_ERR_UNSUPPORTED


def test_validation_returns_before_any_gpu_work(ks):
    lib = ks.raw_library()
    F32, SUM, AFF = ks.DTYPES["f32"], ks.OPS["sum"], ks.OPS["affine_compose"]
    a, b = 0x10000000, 0x20000000   # never dereferenced: every call below fails validation first
    assert lib.ks_scan(99, SUM, 1, a, b, 10, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan(F32, 99, 1, a, b, 10, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan(F32, AFF, 1, a, b, 10, None) == ks.KS_ERR_UNSUPPORTED
    assert lib.ks_scan(F32, SUM, 1, None, b, 10, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan(F32, SUM, 1, a, None, 10, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan(F32, SUM, 1, a + 2, b, 10, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan(ks.DTYPES["u64"], SUM, 1, a + 4, b, 10, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan(F32, SUM, 1, a, a + 8, 10, None) == ks.KS_ERR_OVERLAP
    assert lib.ks_scan(F32, SUM, 1, a + 8, a, 10, None) == ks.KS_ERR_OVERLAP
    assert lib.ks_scan(F32, SUM, 1, None, None, 0, None) == ks.KS_OK          # n == 0: no-op
    assert lib.ks_scan(F32, SUM, 1, a, b, (1 << 40) + 1, None) == ks.KS_ERR_INVALID_ARG
    # with_temp: scratch problems are reported before any launch
    need = lib.ks_scan_temp_bytes(F32, SUM, 1, 1 << 20)
    assert need >= 256 and need % 256 == 0
    assert lib.ks_scan_with_temp(F32, SUM, 1, 1, a, b, 1 << 20, None, need, None) == ks.KS_ERR_WORKSPACE
    assert lib.ks_scan_with_temp(F32, SUM, 1, 1, a, b, 1 << 20, 0x30000000, need - 1, None) == ks.KS_ERR_WORKSPACE
    assert lib.ks_scan_with_temp(F32, SUM, 1, 1, a, b, 1 << 20, 0x30000010, need, None) == ks.KS_ERR_WORKSPACE
    assert lib.ks_scan_with_temp(F32, SUM, 1, 7, a, b, 1 << 20, 0x30000000, need, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_scan_with_temp(F32, SUM, 1, 1, None, None, 0, None, 0, None) == ks.KS_OK
    assert lib.ks_copy(a, a + 16, 64, None) == ks.KS_ERR_OVERLAP
    assert lib.ks_copy(a, b, 60, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_copy(None, None, 0, None) == ks.KS_OK


def test_temp_bytes_grow_with_n_and_cover_both_strategies(ks):
    for dt, op in [("f32", "sum"), ("u64", "sum"), ("argmax_i32_cnt64", "argmax_count")]:
        last = 0
        for k in range(10, 31, 4):
            lb = ks.ks_scan_temp_bytes(dtype=dt, op=op, n=1 << k, algo="lookback")
            rts = ks.ks_scan_temp_bytes(dtype=dt, op=op, n=1 << k, algo="reduce_then_scan")
            auto = ks.ks_scan_temp_bytes(dtype=dt, op=op, n=1 << k)
            assert lb % 256 == 0 and rts % 256 == 0 and lb >= 256 and rts >= 256
            assert auto in (lb, rts)
            assert lb >= last
            last = lb
    assert ks.raw_library().ks_scan_temp_bytes(99, 0, 0, 100) == 0


def test_options_are_validated(ks):
    assert ks.ks_get_option("spin_limit") > 0
    ks.ks_set_option("rows", 8)
    assert ks.ks_get_option("rows") == 8
    ks.ks_set_option("rows", 0)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("rows", 3)
    ks.ks_set_option("waves", 16)
    assert ks.ks_get_option("waves") == 16
    ks.ks_set_option("waves", 0)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("waves", 2)
    for read_only in ("last_grid", "last_wgs_per_cu", "last_waves", "last_rows", "last_form", "last_tickets"):
        assert ks.ks_get_option(read_only) >= 0
        with pytest.raises(ks.KsError):
            ks.ks_set_option(read_only, 1)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("no_such_option", 1)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("tickets", 0)        # by index is not safe for every grid: only -1 (default) and 1
    ks.ks_set_option("tickets", 1)
    assert ks.ks_get_option("tickets") == 1
    ks.ks_set_option("tickets", -1)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("wgs_per_cu", 65)
    ks.ks_set_option("form", 2)
    assert ks.ks_get_option("form") == 2
    ks.ks_set_option("form", -1)
    with pytest.raises(ks.KsError):
        ks.ks_set_option("form", 3)
    assert ks.ks_get_option("no_such_option") == -1


def test_status_strings(ks):
    lib = ks.raw_library()
    seen = {lib.ks_status_string(s) for s in range(0, -8, -1)}
    assert len(seen) == 8
    assert b"gfx950" in lib.ks_version()
