"""GPU parity: the HIP library, called through its C ABI, against the sequential CPU oracle on the
same seeded inputs.  Bars are in tests/parity.py (bit-exact integers / structs; relative 1e-4,
absolute 1e-3 near zero, for floating point against the fp64 oracle)."""
import sys

import numpy as np
import pytest
import torch

import ks_inputs
import oracle
from parity import FLOAT_TOL as FLOAT_TOL_PAIRS
from parity import KINDS, assert_matches, random_input, reference, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    yield ks
    for name, v in [("waves", 0), ("rows", 0), ("prefetch", -1), ("form", -1), ("tickets", -1), ("wgs_per_cu", 0),
                    ("spin_limit", 1 << 20)]:
        ks.ks_set_option(name, v)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def tile_elems(ks, dtype, waves, rows, lookback=True):
    # in the 16-wave look-back kernel one wave of the workgroup holds no data
    data_waves = waves - 1 if (lookback and waves >= 16) else waves
    return data_waves * 64 * rows * 16 // ks.ks_elem_bytes(dtype)


SMALL_INPUT_BYTES = 8 << 20   # up to here the default look-back shape of 4- and 8-byte elements is SMALL_SHAPE
SMALL_SHAPE = (4, 8)


MID_SHAPE = (8, 8)            # between SMALL_INPUT_BYTES and 16 MiB (not for the affine type)


def default_shape(ks, dtype, n=None, op="sum"):
    """(waves, rows) the library picks for the look-back kernel of this element type and size."""
    eb = ks.ks_elem_bytes(dtype)
    if eb not in (4, 8, 16):      # other sizes: the blocked arrangement, rows such that a lane holds whole elements
        return (16, 9) if 144 % eb == 0 else (16, 8)
    if n is not None and eb >= 16 and n * eb <= (1 << 20):
        return 4, 4
    if n is not None and eb < 16:
        if n * eb <= SMALL_INPUT_BYTES:
            return SMALL_SHAPE
        if n * eb <= (16 << 20) and dtype != "affine_f32":
            return MID_SHAPE
    waves, rows = (16, 8) if dtype in ("i64", "u64", "f64") and op == "sum" else (16, 9)
    # up to three rounds of 256 default tiles: the rows that minimise rounds x rows, the default on a
    # tie (16 rows only for one round; the affine type's registers allow neither 12 nor 16 rows)
    if n is not None and eb < 16 and dtype != "affine_f32":
        rounds = lambda r: -(-(-(-n // tile_elems(ks, dtype, waves, r))) // 256)
        if rounds(rows) <= 3:
            best, cost = rows, rounds(rows) * rows
            for cand in ([9] if rows == 8 else []) + [12] + ([16] if rounds(16) == 1 else []) + ([8] if eb == 4 else []):
                if rounds(cand) * cand < cost:
                    best, cost = cand, rounds(cand) * cand
            rows = best
    return waves, rows


RTS_SHAPE = (4, 4)   # tile of the reduce-then-scan kernels


def run(ks, dtype, op, x, inclusive=True, algo="auto", api="with_temp", in_place=False):
    d_in = to_device(x)
    d_out = d_in if in_place else torch.empty_like(d_in)
    n = len(x)
    if api == "plain":
        ks.ks_scan(d_in, d_out, dtype=dtype, op=op, inclusive=inclusive)
    else:
        nbytes = ks.ks_scan_temp_bytes(dtype=dtype, op=op, n=n, algo=algo)
        temp = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        temp.fill_(0xAB)   # previous contents must not matter
        ks.ks_scan_with_temp(d_in, d_out, temp, dtype=dtype, op=op, inclusive=inclusive, algo=algo)
    ks.ks_scan_check()
    return to_host(d_out, x.dtype)


def edge_sizes(*tiles):
    s = {1, 2, 3, 63, 64, 65, 255, 256, 257, 1023, 1025}
    for tile in tiles:   # around one tile, the 64-tile look-back window and two windows
        s |= {tile - 1, tile, tile + 1, 2 * tile + 17, 64 * tile - 1, 64 * tile, 64 * tile + 1, 65 * tile + 3,
              130 * tile + 777}
    return sorted(s)


ALL_PAIRS = sorted(KINDS)


@pytest.mark.parametrize("dtype,op", ALL_PAIRS)
def test_every_pair_edge_sizes_both_strategies(ks, dtype, op):
    for n in edge_sizes(tile_elems(ks, dtype, *default_shape(ks, dtype, op=op)), tile_elems(ks, dtype, *SMALL_SHAPE),
                        tile_elems(ks, dtype, *RTS_SHAPE, lookback=False)):
        x = random_input(dtype, op, n, seed=1000 + n % 97)
        for inclusive in (True, False):
            ref = reference(dtype, op, x, inclusive)
            for algo in ("lookback", "reduce_then_scan", "auto"):
                say(f"[case] pair=({dtype},{op}) n={n} inclusive={inclusive} algo={algo} api=with_temp")
                got = run(ks, dtype, op, x, inclusive, algo)
                assert_matches(dtype, op, got, ref, f"({dtype},{op}) n={n} incl={inclusive} {algo}")


@pytest.mark.parametrize("dtype,op", [("i32", "sum"), ("f32", "sum"), ("u64", "sum"),
                                      ("affine_f32", "affine_compose"), ("argmax_i32_cnt64", "argmax_count"),
                                      ("mat2_u32", "mat2_mul")])
def test_library_owned_workspace_back_to_back(ks, dtype, op):
    # ks_scan: epoch-tagged descriptors reused call after call, sizes going up and down
    tile = tile_elems(ks, dtype, *RTS_SHAPE, lookback=False)
    for n in [300 * tile + 5, 7 * tile, 4000 * tile + 1, 3, 2 * tile, 3999 * tile + 63]:
        x = random_input(dtype, op, n, seed=n % 1013)
        for inclusive in (True, False):
            say(f"[case] pair=({dtype},{op}) n={n} inclusive={inclusive} api=plain")
            got = run(ks, dtype, op, x, inclusive, api="plain")
            assert_matches(dtype, op, got, reference(dtype, op, x, inclusive), f"plain ({dtype},{op}) n={n}")


@pytest.mark.parametrize("dtype,op", [("i32", "sum"), ("f64", "sum"), ("argmax_i32_cnt64", "argmax_count")])
def test_default_shape_switches_with_the_input_size(ks, dtype, op):
    # at and just above the size where the default look-back shape changes from small to large tiles
    at = SMALL_INPUT_BYTES // ks.ks_elem_bytes(dtype)
    mid = (16 << 20) // ks.ks_elem_bytes(dtype)
    tiny16 = (1 << 20) // 16
    for n in (tiny16, tiny16 + 1, at - 1, at, at + 1, mid, mid + 1):
        x = random_input(dtype, op, n, seed=77)
        ref = reference(dtype, op, x, True)
        say(f"[case] pair=({dtype},{op}) n={n} default shape at the small-input limit")
        got = run(ks, dtype, op, x, algo="lookback")
        # both tile counts are below the number of resident workgroups, so the grid tells the tile size
        tile = tile_elems(ks, dtype, *default_shape(ks, dtype, n))
        assert ks.ks_get_option("last_grid") == -(-n // tile), (n, tile)
        assert_matches(dtype, op, got, ref, f"({dtype},{op}) n={n}")


@pytest.mark.parametrize("dtype,op,tiles9,rows", [("i32", "sum", 300, 12), ("f32", "sum", 290, 12),
                                                  ("f32", "sum", 200, 8), ("f32", "sum", 250, 9),
                                                  ("f32", "sum", 400, 16), ("f32", "sum", 500, 9),
                                                  ("f32", "sum", 560, 12), ("f32", "sum", 700, 9),
                                                  ("u64", "sum", 300, 12), ("u64", "sum", 400, 8),
                                                  ("u64", "sum", 470, 9), ("f64", "sum", 470, 9),
                                                  ("u64", "sum", 900, 8), ("affine_f32", "affine_compose", 300, 9)])
def test_inputs_of_a_few_rounds_take_the_rows_that_fill_their_rounds(ks, dtype, op, tiles9, rows):
    # up to three rounds of 256 default tiles the library takes the rows per thread that minimise
    # rounds x rows (12 or 16 rows to fit one round, 12 instead of 9 or 9 instead of 8 to save a
    # round); types whose registers do not allow more rows, and everything longer, keep the default
    n = tiles9 * tile_elems(ks, dtype, 16, 9) - 5
    x = random_input(dtype, op, n, seed=91)
    say(f"[case] pair=({dtype},{op}) n={n}: {tiles9} tiles of 9 rows, expecting {rows} rows")
    assert default_shape(ks, dtype, n) == (16, rows)
    got = run(ks, dtype, op, x, api="plain")
    tiles = -(-n // tile_elems(ks, dtype, 16, rows))
    assert ks.ks_get_option("last_rows") == rows and ks.ks_get_option("last_waves") == 16
    assert ks.ks_get_option("last_grid") == min(tiles, 256), (tiles, ks.ks_get_option("last_grid"))
    assert_matches(dtype, op, got, reference(dtype, op, x, True), f"({dtype},{op}) n={n}")


def test_closed_forms_on_the_gpu(ks):
    n = (1 << 22) + 12345
    say("[case] all-ones int32 / uint64 / f32, iota uint64")
    ones = np.ones(n, dtype=np.int32)
    assert np.array_equal(run(ks, "i32", "sum", ones), np.arange(1, n + 1, dtype=np.int32))
    got = run(ks, "u64", "sum", np.ones(n, dtype=np.uint64), inclusive=False)
    assert np.array_equal(got, np.arange(0, n, dtype=np.uint64))
    # float32 all-ones is exact while the running sum stays below 2^24
    got = run(ks, "f32", "sum", np.ones(n, dtype=np.float32))
    assert np.array_equal(got, np.arange(1, n + 1, dtype=np.float32))
    i = np.arange(n, dtype=np.uint64)
    assert np.array_equal(run(ks, "u64", "sum", i), i * (i + 1) // 2)
    # wrap-around: all INT32_MAX
    big = np.full(n, np.iinfo(np.int32).max, dtype=np.int32)
    with np.errstate(over="ignore"):
        assert np.array_equal(run(ks, "i32", "sum", big), np.cumsum(big, dtype=np.int32))


def test_operand_order_is_kept_at_every_level(ks):
    # Fibonacci matrices: any swapped pair of operands or dropped element breaks the closed form
    n = 70 * 1024 + 5
    say("[case] mat2 Fibonacci closed form, mat2 upper/lower triangular alternation")
    x = np.tile(np.array([[1, 1, 1, 0]], dtype=np.uint32), (n, 1))
    got = run(ks, "mat2_u32", "mat2_mul", x, algo="lookback")
    a, b = 1, 0    # F(1), F(0)
    m = (1 << 32) - 1
    for k in range(1, n + 1):
        a, b = (a + b) & m, a          # a = F(k+1), b = F(k)
        if k % 1009 == 0 or k == n:
            assert got[k - 1].tolist() == [a, b, b, (a - b) & m], k
    # alternating non-commuting factors against the oracle, both strategies
    y = np.where((np.arange(n) % 2 == 0)[:, None], np.array([[1, 1, 0, 1]]), np.array([[1, 0, 1, 1]])).astype(np.uint32)
    ref = reference("mat2_u32", "mat2_mul", y, True)
    for algo in ("lookback", "reduce_then_scan"):
        assert_matches("mat2_u32", "mat2_mul", run(ks, "mat2_u32", "mat2_mul", y, algo=algo), ref, algo)


def test_in_place_and_misaligned_pointers(ks):
    for dtype, op in [("i32", "sum"), ("u64", "sum"), ("argmax_i32_cnt64", "argmax_count"), ("mat2_u32", "mat2_mul"),
                      ("mat2_u64", "mat2_mul"), ("range_i32_cnt32", "range_count")]:
        tile = tile_elems(ks, dtype, *default_shape(ks, dtype))
        n = 37 * tile + 11
        x = random_input(dtype, op, n, seed=5)
        ref = reference(dtype, op, x, True)
        say(f"[case] in-place ({dtype},{op}) n={n}")
        assert_matches(dtype, op, run(ks, dtype, op, x, in_place=True, algo="lookback"), ref, "in place lookback")
        assert_matches(dtype, op, run(ks, dtype, op, x, in_place=True, algo="reduce_then_scan"), ref, "in place rts")
        # element-aligned but not 16-byte aligned: slices that start one element in
        say(f"[case] misaligned ({dtype},{op}) n={n - 1}")
        d_all = to_device(x)
        d_in = d_all[1:]
        d_out_all = torch.empty_like(d_all)
        d_out = d_out_all[1:]
        if ks.ks_elem_bytes(dtype) % 16:
            assert d_in.data_ptr() % 16 != 0
        for algo in ("lookback", "reduce_then_scan"):
            temp = torch.empty(ks.ks_scan_temp_bytes(dtype=dtype, op=op, n=n - 1, algo=algo), dtype=torch.uint8, device="cuda")
            ks.ks_scan_with_temp(d_in.contiguous() if not d_in.is_contiguous() else d_in, d_out, temp,
                                 dtype=dtype, op=op, algo=algo)
            ks.ks_scan_check()
            assert_matches(dtype, op, to_host(d_out, x.dtype), reference(dtype, op, x[1:], True), f"misaligned {algo}")


@pytest.mark.parametrize("dtype,op", [("f32", "sum"), ("i32", "max"), ("u64", "sum"), ("affine_f32", "affine_compose"),
                                      ("argmax_i32_cnt64", "argmax_count"), ("mat2_u64", "mat2_mul"),
                                      ("range_i32_cnt32", "range_count")])
def test_output_pointers_off_the_128_byte_lines(ks, dtype, op):
    # the 16-wave kernels move their tiles to the output's line boundaries (tile 0 is cut short);
    # sizes of a few rounds (12 rows), several rounds and a dozen rounds
    tile9 = tile_elems(ks, dtype, 16, 9)
    if ks.ks_elem_bytes(dtype) in (12, 32):
        plan = ((290, [(1, 1)]), (700, [(1, 1), (0, 3), (5, 2)]))     # large elements: keep the host side short
    else:
        plan = ((290, [(1, 1)]), (700, [(1, 1), (0, 3), (5, 2)]), (3300, [(7, 7), (2, 0)]))
    for tiles, offsets in plan:
        n = tiles * tile9 + 11
        x = random_input(dtype, op, n + 8, seed=tiles)
        d_all = to_device(x)
        d_out_all = torch.zeros_like(d_all)
        for off_in, off_out in offsets:
            for inclusive in (True, False):
                say(f"[case] off-line pointers ({dtype},{op}) n={n} in+{off_in} out+{off_out} elements incl={inclusive}")
                d_in, d_out = d_all[off_in:off_in + n], d_out_all[off_out:off_out + n]
                d_out_all.fill_(0x3C)
                ks.ks_scan(d_in, d_out, dtype=dtype, op=op, inclusive=inclusive)
                ks.ks_scan_check()
                got = to_host(d_out, x.dtype)
                assert_matches(dtype, op, got, reference(dtype, op, x[off_in:off_in + n], inclusive),
                               f"off-line ({dtype},{op}) n={n} +{off_in}/+{off_out}")
                # nothing outside the output view is written
                assert bool((d_out_all[:off_out] == 0x3C).all()) and bool((d_out_all[off_out + n:] == 0x3C).all())
    # in place, off the line
    n = 700 * tile9 + 5
    x = random_input(dtype, op, n + 3, seed=5)
    d_all = to_device(x)
    ks.ks_scan(d_all[3:], d_all[3:], dtype=dtype, op=op)
    ks.ks_scan_check()
    assert_matches(dtype, op, to_host(d_all[3:], x.dtype), reference(dtype, op, x[3:], True), "in place, off the line")


@pytest.mark.parametrize("waves,form", [(4, 0), (8, 0), (16, 1), (16, 2)])
@pytest.mark.parametrize("rows", [4, 8, 9, 12, 16])
@pytest.mark.parametrize("prefetch", [0, 1])
def test_lookback_variants(ks, waves, form, rows, prefetch):
    ks.ks_set_option("waves", waves)
    ks.ks_set_option("rows", rows)
    ks.ks_set_option("prefetch", prefetch)
    ks.ks_set_option("form", form)
    ran = 0
    try:
        for dtype, op in [("f32", "sum"), ("i32", "sum"), ("u64", "sum"), ("affine_f32", "affine_compose"),
                          ("argmax_i32_cnt64", "argmax_count"), ("mat2_u32", "mat2_mul")]:
            tile = tile_elems(ks, dtype, waves, rows)
            # > 2 rounds of a 256-workgroup persistent grid, and the 64-tile window boundary
            for n in [tile * 700 + 3, tile * 64 + 1]:
                x = random_input(dtype, op, n, seed=rows * 10 + prefetch)
                for inclusive in (True, False):
                    say(f"[case] waves={waves} form={form} rows={rows} prefetch={prefetch} ({dtype},{op}) n={n} incl={inclusive}")
                    try:
                        got = run(ks, dtype, op, x, inclusive, algo="lookback")
                    except ks.KsError as e:
                        # shapes that do not fit the register file for this type are refused, never run
                        assert e.status == ks.KS_ERR_UNSUPPORTED, e
                        continue
                    ran += 1
                    assert_matches(dtype, op, got, reference(dtype, op, x, inclusive),
                                   f"waves={waves} rows={rows} pf={prefetch}")
    finally:
        ks.ks_set_option("waves", 0)
        ks.ks_set_option("rows", 0)
        ks.ks_set_option("prefetch", -1)
        ks.ks_set_option("form", -1)
    if ran == 0:
        pytest.skip("no element type fits this shape; every call was refused with KS_ERR_UNSUPPORTED")


def test_repeated_launches_give_identical_integer_results(ks):
    # race hunt: same input many times, small resident grid and full grid, exact compare each time
    n = (1 << 24) + 4099
    x = ks_inputs.whole("int32_sum", n)
    ref = reference("i32", "sum", x, True)
    d_in = to_device(x)
    d_out = torch.empty_like(d_in)
    d_ref = to_device(ref)
    for wgs, tickets in ((0, -1), (0, 1), (3, -1)):
        ks.ks_set_option("wgs_per_cu", wgs)
        ks.ks_set_option("tickets", tickets)
        for it in range(25):
            if it % 8 == 0:
                say(f"[case] repeat int32 sum n={n} wgs_per_cu={wgs} tickets={tickets} iteration={it}")
            d_out.zero_()
            ks.ks_scan(d_in, d_out, dtype="i32", op="sum")
            assert torch.equal(d_out, d_ref), (wgs, tickets, it)
        # more than one workgroup per compute unit is only ever run by ticket
        assert ks.ks_get_option("last_tickets") == (1 if tickets == 1 or wgs == 3 else 0)
    ks.ks_set_option("wgs_per_cu", 0)
    ks.ks_set_option("tickets", -1)
    ks.ks_scan_check()


@pytest.mark.parametrize("dtype,op", [("f32", "sum"), ("u64", "sum"), ("argmax_i32_cnt64", "argmax_count"),
                                      ("mat2_u32", "mat2_mul"), ("affine_f32", "affine_compose"), ("mat2_u64", "mat2_mul")])
def test_tiles_by_ticket(ks, dtype, op):
    # Tile assignment by ticket: every default shape forced onto it, grids of one workgroup per compute
    # unit and grids far larger than what can be resident (4 x 1024 threads per compute unit: most
    # workgroups only start when others have left, draw a ticket past the end and leave too), the small
    # shapes with many workgroups per compute unit, sizes from one tile to a dozen rounds.
    tile = tile_elems(ks, dtype, *default_shape(ks, dtype))
    try:
        for waves, wgs in ((0, 0), (0, 4), (4, 0), (8, 6)):
            ks.ks_set_option("waves", waves)
            ks.ks_set_option("wgs_per_cu", wgs)
            ks.ks_set_option("tickets", 1)
            for n in (17, tile + 1, 255 * tile + 3, 257 * tile, 700 * tile + 5, 3100 * tile + 11):
                x = random_input(dtype, op, n, seed=n % 101)
                for inclusive, api in ((True, "with_temp"), (False, "with_temp"), (True, "plain")):
                    if api == "plain" and n <= tile:
                        continue          # ks_scan hands a single tile to one workgroup without any look-back
                    say(f"[case] by ticket ({dtype},{op}) waves={waves} wgs_per_cu={wgs} n={n} incl={inclusive} {api}")
                    try:
                        got = run(ks, dtype, op, x, inclusive, algo="lookback", api=api)
                    except ks.KsError as e:
                        assert e.status == ks.KS_ERR_UNSUPPORTED, e     # shape not compiled for this type
                        continue
                    assert ks.ks_get_option("last_tickets") == 1
                    assert_matches(dtype, op, got, reference(dtype, op, x, inclusive), f"by ticket ({dtype},{op}) n={n}")
    finally:
        for name, v in (("waves", 0), ("wgs_per_cu", 0), ("tickets", -1)):
            ks.ks_set_option(name, v)


def test_abandoned_wait_is_reported_and_the_next_call_is_clean(ks):
    # A spin limit of zero makes the first workgroup that has to wait give up.  Every workgroup must
    # still exit (the call returns), the check reports the timeout once, and later calls are unaffected.
    for dtype, op in [("f32", "sum"), ("u64", "sum"), ("argmax_i32_cnt64", "argmax_count")]:
        tile = tile_elems(ks, dtype, *default_shape(ks, dtype))
        n = 900 * tile + 7
        x = random_input(dtype, op, n, seed=77)
        d_in = to_device(x)
        d_out = torch.empty_like(d_in)
        ks.ks_set_option("spin_limit", 0)
        try:
            say(f"[case] spin_limit=0 ({dtype},{op}) n={n}")
            ks.ks_scan(d_in, d_out, dtype=dtype, op=op)
            try:
                ks.ks_scan_check()
                timed_out = False      # legal: nobody happened to wait
            except ks.KsError as e:
                assert e.status == ks.KS_ERR_TIMEOUT, e
                timed_out = True
            say(f"[done] spin_limit=0 ({dtype},{op}): timed_out={timed_out}")
        finally:
            ks.ks_set_option("spin_limit", 1 << 20)
        ks.ks_scan_check()             # the flag was cleared by the check that reported it
        for api in ("plain", "with_temp"):
            got = run(ks, dtype, op, x, True, algo="lookback", api=api)
            assert_matches(dtype, op, got, reference(dtype, op, x, True), f"after timeout ({dtype},{op}) {api}")


MAP_TRIPLES = [("f32", "square", "sum"), ("f32", "abs", "sum"), ("f32", "abs", "max"), ("f64", "square", "sum"),
               ("i32", "nonzero", "sum"), ("i32", "abs", "max"), ("i32", "square", "sum"), ("u64", "nonzero", "sum")]


@pytest.mark.parametrize("dtype,map_name,op", MAP_TRIPLES)
def test_map_fused_scan(ks, dtype, map_name, op):
    # scan(f, op, src): sizes around the look-back tile, the 64-tile window and the single-workgroup path
    tile = tile_elems(ks, dtype, *default_shape(ks, dtype))
    rts = tile_elems(ks, dtype, *RTS_SHAPE, lookback=False)
    oop, odt, npdt, _ = KINDS[(dtype, op)]
    rng = np.random.default_rng(99)
    for n in [1, 5, rts - 1, rts, rts + 1, tile - 1, tile + 1, 64 * tile + 1, 300 * tile + 12345]:
        if np.issubdtype(npdt, np.integer):
            x = (rng.integers(0, 3, size=n) * rng.integers(-1000, 1000, size=n)).astype(npdt)   # one third zeros
        else:
            x = rng.uniform(-2.0, 2.0, size=n).astype(npdt)
        for inclusive in (True, False):
            say(f"[case] map-fused ({dtype},{map_name},{op}) n={n} inclusive={inclusive}")
            ref = oracle.mapped_scan(map_name, oop, odt, x, inclusive)
            d_in = to_device(x)
            d_out = torch.empty_like(d_in)
            ks.ks_scan_map(d_in, d_out, dtype=dtype, map=map_name, op=op, inclusive=inclusive)
            ks.ks_scan_check()
            got = to_host(d_out, x.dtype)
            if (dtype, op) in FLOAT_TOL_PAIRS:      # float sums: tolerance against the oracle's float64 answer
                assert_matches(dtype, op, got, ref, f"map ({dtype},{map_name},{op}) n={n} incl={inclusive}")
            else:
                assert got.tobytes() == ref.tobytes(), (dtype, map_name, op, n, inclusive,
                                                        int(np.flatnonzero(got != ref)[0]))
    # the identity map is the plain scan
    x = random_input(dtype, op, 3 * tile + 5, seed=3)
    d_in = to_device(x)
    a, b = torch.empty_like(d_in), torch.empty_like(d_in)
    ks.ks_scan_map(d_in, a, dtype=dtype, map="identity", op=op)
    ks.ks_scan(d_in, b, dtype=dtype, op=op)
    ks.ks_scan_check()
    if (dtype, op) in FLOAT_TOL_PAIRS:
        assert torch.allclose(a, b, rtol=1e-4, atol=1e-3)
    else:
        assert torch.equal(a, b)


@pytest.mark.parametrize("dtype,op", [("i32", "sum"), ("f32", "sum"), ("u64", "max"),
                                      ("argmax_i32_cnt64", "argmax_count"), ("mat2_u32", "mat2_mul"),
                                      ("mat2_u64", "mat2_mul"), ("range_i32_cnt32", "range_count")])
def test_strided_views(ks, dtype, op):
    # one column of a row-major [n, stride] matrix in, another layout out; the rest must stay untouched
    rts = tile_elems(ks, dtype, *RTS_SHAPE, lookback=False)
    sizes = [1, 2, rts - 1, rts, rts + 1, 5 * rts + 3]
    if dtype == "i32":
        sizes.append(rts * rts + 5)      # thousands of tiles, several look-back windows
        sizes.append(40_000_003)         # more tiles than any resident grid: every workgroup loops
    for n in sizes:
        for in_stride, out_stride in [(3, 1), (1, 2), (5, 5)]:
            x = random_input(dtype, op, n, seed=n % 89 + in_stride)
            words = ks.ks_elem_bytes(dtype) // 4          # device storage in 32-bit words per element
            host = to_device(x).reshape(n, -1).view(torch.int32).reshape(n, words)
            d_in = torch.full((n, in_stride, words), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            d_in[:, 0, :] = host
            sentinel = 0x3C3C3C3C
            d_out = torch.full((n, out_stride, words), sentinel, dtype=torch.int32, device="cuda")
            for inclusive in (True, False):
                say(f"[case] strided ({dtype},{op}) n={n} strides=({in_stride},{out_stride}) inclusive={inclusive}")
                d_out.fill_(sentinel)
                ks.ks_scan_strided(d_in, d_out, dtype=dtype, op=op, n=n, in_stride=in_stride,
                                   out_stride=out_stride, inclusive=inclusive)
                ks.ks_scan_check()
                got_words = d_out[:, 0, :].contiguous()
                got = to_host(got_words.view(to_device(x).dtype).reshape(to_device(x).shape), x.dtype)
                assert_matches(dtype, op, got, reference(dtype, op, x, inclusive),
                               f"strided ({dtype},{op}) n={n} ({in_stride},{out_stride}) incl={inclusive}")
                if out_stride > 1:
                    assert bool((d_out[:, 1:, :] == sentinel).all()), "elements between the strides were written"
            if in_stride == out_stride:      # the same view in place
                say(f"[case] strided in place ({dtype},{op}) n={n} stride={in_stride}")
                ks.ks_scan_strided(d_in, d_in, dtype=dtype, op=op, n=n, in_stride=in_stride, out_stride=in_stride)
                ks.ks_scan_check()
                got_words = d_in[:, 0, :].contiguous()
                got = to_host(got_words.view(to_device(x).dtype).reshape(to_device(x).shape), x.dtype)
                assert_matches(dtype, op, got, reference(dtype, op, x, True), f"strided in place ({dtype},{op}) n={n}")
                assert bool((d_in[:, 1:, :] == 0x5A5A5A5A).all())


def test_random_pairs_sizes_offsets(ks):
    # seeded sweep over every pair: sizes log-uniform up to 2.5e8 bytes (a third of them above 2e6
    # elements), pointers moved by up to 39 elements, inclusive / exclusive, some in place
    rng = np.random.default_rng(20261127)
    for case in range(240):
        dtype, op = ALL_PAIRS[int(rng.integers(len(ALL_PAIRS)))]
        eb = ks.ks_elem_bytes(dtype)
        lo = np.log(2e6) if case % 3 == 0 else 0.0
        n = int(np.exp(rng.uniform(lo, np.log(2.5e8 / eb))))
        off_in, off_out = (int(rng.integers(0, 40)), int(rng.integers(0, 40))) if rng.random() < 0.6 else (0, 0)
        inclusive = bool(rng.integers(2))
        in_place = rng.random() < 0.2
        if in_place:
            off_out = off_in
        x = random_input(dtype, op, n + 40, seed=int(rng.integers(1 << 30)))
        d_all = to_device(x)
        d_out_all = d_all if in_place else torch.zeros_like(d_all)
        say(f"[case {case}] ({dtype},{op}) n={n} in+{off_in} out+{off_out} incl={inclusive} in_place={in_place}")
        ks.ks_scan(d_all[off_in:off_in + n], d_out_all[off_out:off_out + n], dtype=dtype, op=op, inclusive=inclusive)
        ks.ks_scan_check()
        got = to_host(d_out_all[off_out:off_out + n], x.dtype)
        assert_matches(dtype, op, got, reference(dtype, op, x[off_in:off_in + n], inclusive), f"case {case}")
        del d_all, d_out_all


def test_two_streams_at_once(ks):
    # calls on different streams use different workspaces and may overlap on the device; each stream's
    # results must be those of its own inputs
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    tile = tile_elems(ks, "i32", *default_shape(ks, "i32"))
    n1, n2 = 900 * tile + 17, 700 * tile_elems(ks, "u64", *default_shape(ks, "u64")) + 5
    x1 = ks_inputs.whole("int32_sum", n1)
    x2 = random_input("u64", "sum", n2, seed=21)
    r1, r2 = reference("i32", "sum", x1, True), reference("u64", "sum", x2, False)
    d1, d2 = to_device(x1), to_device(x2)
    o1, o2 = torch.empty_like(d1), torch.empty_like(d2)
    want1, want2 = to_device(r1), to_device(r2)
    torch.cuda.synchronize()
    for it in range(20):
        if it % 5 == 0:
            say(f"[case] two streams, iteration {it}")
        o1.zero_()
        o2.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            ks.ks_scan(d1, o1, dtype="i32", op="sum", inclusive=True)
        with torch.cuda.stream(s2):
            ks.ks_scan(d2, o2, dtype="u64", op="sum", inclusive=False)
        with torch.cuda.stream(s1):
            ks.ks_scan(d1, o1, dtype="i32", op="sum", inclusive=True)
        ks.ks_scan_check(s1)
        ks.ks_scan_check(s2)
        assert torch.equal(o1, want1), it
        assert torch.equal(o2, want2), it


def test_two_host_threads_on_their_own_streams(ks):
    # The library's state (options, per-stream scratch, epochs, abort words) is shared by all host
    # threads; two threads that scan and reduce on streams of their own, at the same time (the binding
    # releases the interpreter lock during a call), must each get the results of their own inputs.
    import threading
    jobs = []
    for k, (dtype, op, n, seed) in enumerate((("i32", "sum", 3_000_017, 31), ("u64", "sum", 1_700_003, 32))):
        x = random_input(dtype, op, n, seed=seed)
        scan_ref = to_device(reference(dtype, op, x, True))
        total = reference(dtype, op, x, True)[-1]
        jobs.append({"dtype": dtype, "op": op, "d_in": to_device(x), "want": scan_ref, "total": int(total),
                     "stream": torch.cuda.Stream(), "errors": []})
    torch.cuda.synchronize()

    def work(job):
        try:
            d_in, s = job["d_in"], job["stream"]
            out = torch.empty_like(d_in)
            one = torch.empty_like(d_in[:1])
            temp = torch.empty(ks.ks_scan_temp_bytes(dtype=job["dtype"], op=job["op"], n=d_in.numel()), dtype=torch.uint8,
                               device="cuda")
            for it in range(60):
                out.zero_()
                one.zero_()
                if it % 3 == 2:
                    ks.ks_scan_with_temp(d_in, out, temp, dtype=job["dtype"], op=job["op"], stream=s)
                else:
                    ks.ks_scan(d_in, out, dtype=job["dtype"], op=job["op"], stream=s)
                ks.ks_mapreduce(d_in, one, dtype=job["dtype"], op=job["op"], stream=s)
                ks.ks_scan_check(s)
                if not torch.equal(out, job["want"]):
                    job["errors"].append(f"scan differs in iteration {it}")
                got = int(to_host(one, np.int32 if job["dtype"] == "i32" else np.uint64)[0])
                if got != job["total"]:
                    job["errors"].append(f"reduction {got} != {job['total']} in iteration {it}")
        except Exception as e:      # a thread's exception would otherwise be lost
            job["errors"].append(repr(e))

    say("[case] two host threads, each with its own stream: 60 scans and reductions each")
    threads = [threading.Thread(target=work, args=(job,)) for job in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for job in jobs:
        assert not job["errors"], job["errors"][:3]


def test_release_scratch(ks):
    # the library-owned scratch of a stream can be given back; the next call allocates again; a
    # buffer that a graph has recorded is kept
    s = torch.cuda.Stream()
    ks.ks_release_scratch(s)                       # nothing cached yet: a no-op
    dtype, op, n = "argmax_i32_cnt64", "argmax_count", 1 << 26
    x = ks_inputs.whole("argmax", 1 << 16)
    d_in = to_device(x).repeat(n >> 16, 1)
    d_out = torch.empty_like(d_in)
    small = random_input("i32", "sum", 100_003, seed=9)
    d_small, ref_small = to_device(small), to_device(reference("i32", "sum", small, True))
    o_small = torch.empty_like(d_small)
    expect = ks.ks_scan_temp_bytes(dtype=dtype, op=op, n=n)
    assert expect >= 4 << 20
    torch.cuda.synchronize()
    say(f"[case] release scratch: {expect} bytes held by a stream, then given back")
    free_before = torch.cuda.mem_get_info()[0]
    ks.ks_scan(d_in, d_out, dtype=dtype, op=op, stream=s)
    ks.ks_scan_check(s)
    free_held = torch.cuda.mem_get_info()[0]
    ks.ks_release_scratch(s)
    free_released = torch.cuda.mem_get_info()[0]
    assert free_before - free_held >= expect // 2, (free_before, free_held, expect)
    assert free_released - free_held >= expect // 2, (free_released, free_held, expect)
    for _ in range(2):                             # allocates again (the smallest buffer), then reuses it
        o_small.zero_()
        ks.ks_scan(d_small, o_small, dtype="i32", op="sum", stream=s)
        ks.ks_scan_check(s)
        assert torch.equal(o_small, ref_small)
    # recorded into a graph: the release leaves the buffer alone and the replays stay right
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        ks.ks_scan(d_small, o_small, dtype="i32", op="sum")
    ks.ks_release_scratch(s)
    for _ in range(3):
        o_small.zero_()
        with torch.cuda.stream(s):
            graph.replay()
        ks.ks_scan_check(s)
        assert torch.equal(o_small, ref_small)
    del graph


def test_hip_graph_replays_match_eager_results(ks):
    # ks_scan_with_temp allocates nothing and clears its descriptors with a kernel, so a caller may
    # record it into a HIP graph (after one eager call, which runs the one-off residency check of
    # the kernel variant).  Every replay, with fresh input contents and eager work in between, must
    # give what the eager call gives for the same input.
    for dtype, op, n in (("f32", "sum", 3_000_017), ("u64", "sum", 1_500_003), ("i32", "max", 70_001)):
        xs = [random_input(dtype, op, n, seed=40 + r) for r in range(4)]
        refs = [reference(dtype, op, x, True) for x in xs]
        d_in = to_device(xs[0])
        d_out = torch.empty_like(d_in)
        temp = torch.empty(ks.ks_scan_temp_bytes(dtype=dtype, op=op, n=n, algo="lookback"), dtype=torch.uint8,
                           device="cuda")
        say(f"[case] hip graph ({dtype},{op}) n={n}: eager warm-up")
        ks.ks_scan_with_temp(d_in, d_out, temp, dtype=dtype, op=op, inclusive=True, algo="lookback")
        ks.ks_scan_check()
        assert_matches(dtype, op, to_host(d_out, xs[0].dtype), refs[0], "eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ks.ks_scan_with_temp(d_in, d_out, temp, dtype=dtype, op=op, inclusive=True, algo="lookback")
        for r in range(4):
            say(f"[case] hip graph ({dtype},{op}) n={n}: replay {r}")
            d_in.copy_(to_device(xs[r]))
            d_out.zero_()
            temp.fill_(0x5A + r)          # eager work on the buffers between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ks.ks_scan_check()
            assert_matches(dtype, op, to_host(d_out, xs[r].dtype), refs[r], f"replay {r}")
        del graph


def test_ks_scan_recorded_into_a_graph(ks):
    # ks_scan with its library-owned scratch under stream capture: a replay repeats the kernel
    # arguments of the recording, epoch included, so the recorded call must not rely on the epoch to
    # tell its descriptors from those the previous replay (or an eager call in between) left behind.
    for dtype, op, n in (("f32", "sum", 3_000_017), ("argmax_i32_cnt64", "argmax_count", 1_200_003)):
        xs = [random_input(dtype, op, n, seed=60 + r) for r in range(4)]
        refs = [reference(dtype, op, x, True) for x in xs]
        side = random_input(dtype, op, n // 2 + 7, seed=59)
        side_ref = reference(dtype, op, side, True)
        d_in = to_device(xs[0])
        d_out = torch.empty_like(d_in)
        d_side, d_side_out = to_device(side), torch.empty_like(to_device(side))
        # the scratch belongs to (device, stream): warm up, record and replay on one stream
        s = torch.cuda.Stream()
        torch.cuda.synchronize()
        say(f"[case] ks_scan in a graph ({dtype},{op}) n={n}: eager warm-up (allocates the scratch)")
        with torch.cuda.stream(s):
            ks.ks_scan(d_in, d_out, dtype=dtype, op=op)
        ks.ks_scan_check(s)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            ks.ks_scan(d_in, d_out, dtype=dtype, op=op)
        for r in range(4):
            say(f"[case] ks_scan in a graph ({dtype},{op}) n={n}: replay {r}")
            d_in.copy_(to_device(xs[r]))
            d_out.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(s):
                # eager calls on the same stream and scratch between the replays
                ks.ks_scan(d_side, d_side_out, dtype=dtype, op=op)
                graph.replay()
                graph.replay()             # twice in a row: the second finds the first one's descriptors
            ks.ks_scan_check(s)
            assert_matches(dtype, op, to_host(d_out, xs[r].dtype), refs[r], f"replay {r}")
            assert_matches(dtype, op, to_host(d_side_out, side.dtype), side_ref, f"eager call before replay {r}")
        # a recording that would have to allocate is refused, not attempted
        big = torch.zeros(64 * n * (d_in.numel() // n), dtype=d_in.dtype, device="cuda")
        big_out = torch.empty_like(big)
        g2 = torch.cuda.CUDAGraph()
        refused = False
        with torch.cuda.graph(g2, stream=s):
            try:
                ks.ks_scan(big, big_out, dtype=dtype, op=op)
            except ks.KsError as e:
                assert e.status == ks.KS_ERR_WORKSPACE, e
                refused = True
        assert refused
        del graph, g2, big, big_out


def test_a_timeout_is_reported_on_the_stream_it_happened_on(ks):
    # abort words are per stream: a wait abandoned on stream A is reported by the check of A and
    # not by the check of B, and scans on B meanwhile are unaffected
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    tile = tile_elems(ks, "u64", 16, 8)
    n = 900 * tile + 7
    x = random_input("u64", "sum", n, seed=3)
    ref = to_device(reference("u64", "sum", x, True))
    d_in = to_device(x)
    out_a, out_b = torch.empty_like(d_in), torch.empty_like(d_in)
    with torch.cuda.stream(sa), torch.cuda.stream(sb):
        pass
    torch.cuda.synchronize()
    seen = 0
    for it in range(5):
        ks.ks_set_option("spin_limit", 0)
        try:
            with torch.cuda.stream(sa):
                ks.ks_scan(d_in, out_a, dtype="u64", op="sum")
        finally:
            ks.ks_set_option("spin_limit", 1 << 20)
        with torch.cuda.stream(sb):
            ks.ks_scan(d_in, out_b, dtype="u64", op="sum")
        ks.ks_scan_check(sb)                       # must not raise: B's scans never gave up
        assert torch.equal(out_b, ref), it
        try:
            ks.ks_scan_check(sa)
        except ks.KsError as e:
            assert e.status == ks.KS_ERR_TIMEOUT, e
            seen += 1
        ks.ks_scan_check(sa)                       # reported once, then clear
        say(f"[case] per-stream abort word, iteration {it}: timeouts seen on A so far {seen}")
    assert seen >= 1, "with a spin limit of zero some workgroup of 900 tiles has to wait at least once in five runs"


@pytest.mark.parametrize("tickets", [-1, 1])
def test_scan_while_another_stream_holds_the_compute_units(ks, tickets):
    # A bounded queue of plain copies on another stream keeps the compute units busy while the scan
    # is launched, so its workgroups start late and not together.  The scan must come out right, or
    # its own stream's check must say KS_ERR_TIMEOUT; every kernel ends by itself either way.
    other = torch.cuda.Stream()
    n = 1 << 26
    x = ks_inputs.whole("int32_sum", n)
    want = to_device(reference("i32", "sum", x, True))
    d_in = to_device(x)
    d_out = torch.empty_like(d_in)
    a = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    ks.ks_set_option("tickets", tickets)
    try:
        ks.ks_scan(d_in, d_out, dtype="i32", op="sum")      # warm-up: scratch allocated, clocks up
        torch.cuda.synchronize()
        outcomes = {"ok": 0, "timeout": 0}
        for it in range(6):
            d_out.zero_()
            torch.cuda.synchronize()
            with torch.cuda.stream(other):
                for _ in range(40):                         # about 4 ms of copies
                    ks.ks_copy(a, b, stream=other)
            for _ in range(3):                              # three scans land in the middle of them
                ks.ks_scan(d_in, d_out, dtype="i32", op="sum")
            try:
                ks.ks_scan_check()
                assert torch.equal(d_out, want), f"iteration {it}: wrong result without a reported timeout"
                outcomes["ok"] += 1
            except ks.KsError as e:
                assert e.status == ks.KS_ERR_TIMEOUT, e
                outcomes["timeout"] += 1
            other.synchronize()
        say(f"[case] scan beside a queue of copies, tickets={tickets}: {outcomes}")
        if tickets == 1:
            assert outcomes["timeout"] == 0      # by ticket nobody ever waits for a workgroup that has not started
    finally:
        ks.ks_set_option("tickets", -1)
    ks.ks_scan_check()


def test_more_than_2_pow_32_elements(ks):
    # 64-bit index arithmetic end to end: all-ones int32, closed form out[i] = i + 1 (mod 2^32), checked
    # on the device chunk by chunk (16 GiB in, 16 GiB out; the sums wrap exactly once, at element 2^32 - 1)
    n = (1 << 32) + 12345
    say(f"[case] int32 all-ones n={n} (> 2^32 elements)")
    d_in = torch.ones(n, dtype=torch.int32, device="cuda")
    d_out = torch.empty_like(d_in)
    ks.ks_scan(d_in, d_out, dtype="i32", op="sum")
    ks.ks_scan_check()
    step = 1 << 28
    for at in range(0, n, step):
        m = min(step, n - at)
        want = (torch.arange(at + 1, at + 1 + m, dtype=torch.int64, device="cuda") & 0xFFFFFFFF)
        got = d_out[at:at + m].to(torch.int64) & 0xFFFFFFFF
        assert torch.equal(got, want), f"mismatch in chunk at {at}"
    del d_in, d_out
    torch.cuda.empty_cache()


# ---------------------------------------------------------------- the five benchmark configurations, full size

def _full_config(ks, name, n=None, api="plain", algo="auto"):
    """Stream the workload to the device chunk by chunk, scan it in one call, compare chunk by chunk."""
    w = ks_inputs.WORKLOADS[name]
    n = w.n if n is None else n
    oop, odt, npdt, cols = KINDS[(w.dtype, w.op)]
    host_cols = 4 if npdt == oracle.ARGMAX_DTYPE else cols
    tdt = {np.dtype(np.int32): torch.int32, np.dtype(np.float32): torch.float32,
           np.dtype(np.uint64): torch.int64}.get(np.dtype(npdt), torch.int32)
    shape = (n,) if host_cols == 1 else (n, host_cols)
    d_in = torch.empty(shape, dtype=tdt, device="cuda")
    at = 0
    for chunk in ks_inputs.chunks(name, n):
        d_in[at:at + len(chunk)] = to_device(chunk)
        at += len(chunk)
    d_out = torch.empty_like(d_in)
    say(f"[case] workload={name} n={n} api={api} algo={algo}")
    if api == "plain":
        ks.ks_scan(d_in, d_out, dtype=w.dtype, op=w.op, inclusive=w.inclusive)
    else:
        temp = torch.empty(ks.ks_scan_temp_bytes(dtype=w.dtype, op=w.op, n=n, algo=algo), dtype=torch.uint8, device="cuda")
        ks.ks_scan_with_temp(d_in, d_out, temp, dtype=w.dtype, op=w.op, inclusive=w.inclusive, algo=algo)
    ks.ks_scan_check()
    stream = oracle.ScanStream(oop, odt, w.inclusive)
    worst, at = 0.0, 0
    for chunk in ks_inputs.chunks(name, n):
        ref = stream.feed(chunk)
        got = to_host(d_out[at:at + len(chunk)], chunk.dtype)
        worst = max(worst, assert_matches(w.dtype, w.op, got, ref, f"{name} n={n} chunk at {at}"))
        at += len(chunk)
    say(f"[done] workload={name} n={n}: worst float ratio {worst:.4f}")
    return worst


def test_config_int32_sum_2_20(ks):
    _full_config(ks, "int32_sum")
    _full_config(ks, "int32_sum", api="with_temp", algo="lookback")
    _full_config(ks, "int32_sum", api="with_temp", algo="reduce_then_scan")


def test_config_f32_sum_2_28(ks):
    assert _full_config(ks, "f32_sum") <= 1.0
    assert _full_config(ks, "f32_sum", api="with_temp", algo="reduce_then_scan") <= 1.0


def test_f32_sum_2_28_is_exact_on_small_integers(ks):
    # The float bar at the end of config 2 is 1e-4 x 1.3e8: a dropped or doubled element would pass it.
    # Inputs in {0, 1} with a total below 2^24 make every partial sum an integer that float32 holds
    # exactly, whatever the order of the additions, so the default kernel of the headline size (and the
    # fallback) must reproduce the oracle bit for bit at all 2^28 positions.
    n = 1 << 28
    rng = np.random.default_rng(28)
    d_in = torch.empty(n, dtype=torch.float32, device="cuda")
    d_ref = torch.empty(n, dtype=torch.float32, device="cuda")
    stream = oracle.ScanStream("sum", "f32", True)
    total = 0.0
    for at in range(0, n, ks_inputs.CHUNK):
        x = (rng.random(ks_inputs.CHUNK, dtype=np.float32) < 0.05).astype(np.float32)
        ref = stream.feed(x)
        total = float(ref[-1])
        d_in[at:at + len(x)] = torch.from_numpy(x).cuda()
        d_ref[at:at + len(x)] = torch.from_numpy(ref.astype(np.float32)).cuda()
    assert total < float(1 << 24), total
    d_out = torch.empty_like(d_in)
    for inclusive in (True, False):
        say(f"[case] f32 sum n=2^28, inputs in {{0,1}}, total {total:.0f}, inclusive={inclusive}: exact compare")
        ks.ks_scan(d_in, d_out, dtype="f32", op="sum", inclusive=inclusive)
        ks.ks_scan_check()
        assert ks.ks_get_option("last_waves") == 16 and ks.ks_get_option("last_rows") == 9
        if inclusive:
            assert torch.equal(d_out, d_ref)
        else:
            assert float(d_out[0]) == 0.0 and torch.equal(d_out[1:], d_ref[:-1])
    temp = torch.empty(ks.ks_scan_temp_bytes(dtype="f32", op="sum", n=n, algo="reduce_then_scan"), dtype=torch.uint8,
                       device="cuda")
    say("[case] f32 sum n=2^28, inputs in {0,1}, reduce-then-scan: exact compare")
    ks.ks_scan_with_temp(d_in, d_out, temp, dtype="f32", op="sum", inclusive=True, algo="reduce_then_scan")
    ks.ks_scan_check()
    assert torch.equal(d_out, d_ref)


def test_config_u64_exclusive_sum_2_27(ks):
    _full_config(ks, "u64_exsum")
    _full_config(ks, "u64_exsum", api="with_temp", algo="reduce_then_scan")


def test_config_affine_2_26(ks):
    assert _full_config(ks, "affine") <= 1.0
    assert _full_config(ks, "affine", api="with_temp", algo="reduce_then_scan") <= 1.0


@pytest.mark.parametrize("log2n", list(range(10, 29, 2)))
def test_config_argmax_struct_sweep(ks, log2n):
    _full_config(ks, "argmax", n=1 << log2n)
    _full_config(ks, "argmax", n=1 << log2n, api="with_temp", algo="reduce_then_scan")


def test_config_argmax_struct_2_30(ks):
    _full_config(ks, "argmax", n=1 << 30)
