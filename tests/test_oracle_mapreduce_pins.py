"""Pins of the oracle's mapreduce (CPU only): op(f(x_1), ..., f(x_n)) of the paper's Sec. II-C / V-A.

What fixes it, other than itself: library reductions (numpy sum / min / max / count_nonzero with
the wrap of the element type), exact sums (math.fsum, Python integers, rationals), closed forms,
the definition of the arg-max struct, brute force over every order of the elements for the
commutative operators and over every parenthesisation for the others, on tiny inputs."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import ks_inputs
import oracle

INT_TYPES = ["i32", "u32", "i64", "u64"]
NP = {"i32": np.int32, "u32": np.uint32, "i64": np.int64, "u64": np.uint64, "f32": np.float32, "f64": np.float64}
BITS = {"i32": 32, "u32": 32, "i64": 64, "u64": 64}


def wrap(value: int, dt: str) -> int:
    bits = BITS[dt]
    value &= (1 << bits) - 1
    if dt.startswith("i") and value >= 1 << (bits - 1):
        value -= 1 << bits
    return value


@pytest.mark.parametrize("dt", INT_TYPES)
def test_integer_sum_is_the_exact_sum_modulo_2w(dt):
    rng = np.random.default_rng(3)
    info = np.iinfo(NP[dt])
    x = rng.integers(info.min, info.max, size=100_003, dtype=NP[dt], endpoint=True)
    exact = sum(int(v) for v in x)                      # Python integers: no wrap
    assert int(oracle.mapreduce("identity", "sum", dt, x)) == wrap(exact, dt)
    # closed forms: all ones, and 0 .. n-1
    n = 70_001
    assert int(oracle.mapreduce("identity", "sum", dt, np.ones(n, NP[dt]))) == n
    assert int(oracle.mapreduce("identity", "sum", dt, np.arange(n).astype(NP[dt]))) == wrap(n * (n - 1) // 2, dt)


@pytest.mark.parametrize("dt", INT_TYPES + ["f32", "f64"])
def test_min_and_max_are_numpy_min_and_max(dt):
    rng = np.random.default_rng(4)
    x = (rng.normal(size=50_001) * 1e6).astype(NP[dt]) if dt in ("f32", "f64") else \
        rng.integers(np.iinfo(NP[dt]).min, np.iinfo(NP[dt]).max, size=50_001, dtype=NP[dt], endpoint=True)
    assert oracle.mapreduce("identity", "min", dt, x) == x.min()
    assert oracle.mapreduce("identity", "max", dt, x) == x.max()
    # chunks smaller than the input change nothing
    assert oracle.mapreduce("identity", "max", dt, x, chunk=777) == x.max()


@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_float_sum_against_the_exact_sum(dt):
    rng = np.random.default_rng(5)
    n = 200_003
    x = rng.uniform(-1.0, 1.0, size=n).astype(NP[dt])
    exact = math.fsum(float(v) for v in x)              # correctly rounded sum of the stored values
    got = float(oracle.mapreduce("identity", "sum", dt, x))
    # a float64 (long double for float64 inputs) fold of n values bounded by 1: error below n * 2^-53 * max partial sum
    assert abs(got - exact) <= n * 2.0 ** -53 * max(1.0, np.abs(np.cumsum(x.astype(np.float64))).max())
    # and it is NOT the float32 answer for float32 inputs: the fold runs one precision step above the input
    if dt == "f32":
        big = np.ones(1 << 25, np.float32)
        assert float(oracle.mapreduce("identity", "sum", "f32", big)) == float(1 << 25)    # a float32 fold stalls at 2^24


def test_maps_square_abs_nonzero():
    rng = np.random.default_rng(6)
    n = 30_001
    i = np.arange(1, n + 1)
    # sum of squares 1^2 + ... + n^2 = n (n + 1) (2n + 1) / 6, mod 2^32 for int32
    want = n * (n + 1) * (2 * n + 1) // 6
    assert int(oracle.mapreduce("square", "sum", "i32", i.astype(np.int32))) == wrap(want, "i32")
    assert float(oracle.mapreduce("square", "sum", "f64", i.astype(np.float64))) == float(want)   # exact below 2^53
    xf = rng.uniform(-3, 3, size=n).astype(np.float32)
    exact = math.fsum(float(v) * float(v) for v in xf)  # float32 squares are exact in float64
    assert abs(float(oracle.mapreduce("square", "sum", "f32", xf)) - exact) <= 1e-9 * exact
    assert float(oracle.mapreduce("abs", "max", "f32", xf)) == float(np.abs(xf).max())
    assert float(oracle.mapreduce("abs", "sum", "f32", xf)) == pytest.approx(math.fsum(abs(float(v)) for v in xf), rel=1e-12)
    xi = (rng.integers(0, 3, size=n) * rng.integers(-9, 9, size=n)).astype(np.int32)
    assert int(oracle.mapreduce("nonzero", "sum", "i32", xi)) == int(np.count_nonzero(xi))
    assert int(oracle.mapreduce("abs", "max", "i32", xi)) == int(np.abs(xi).max())
    assert int(oracle.mapreduce("nonzero", "sum", "u64", xi.astype(np.int64).view(np.uint64))) == int(np.count_nonzero(xi))


def test_empty_and_single_element():
    for dt in INT_TYPES + ["f32", "f64"]:
        assert oracle.mapreduce("identity", "sum", dt, np.zeros(0, NP[dt])) == 0
        e = np.zeros(0, NP[dt])
        big, small = oracle.mapreduce("identity", "min", dt, e), oracle.mapreduce("identity", "max", dt, e)
        probe = np.array([5, 1, 9]).astype(NP[dt])
        assert all(min(big, v) == v and max(small, v) == v for v in probe)      # identities of min and max
        assert oracle.mapreduce("square", "sum", dt, np.array([7]).astype(NP[dt])) == 49
    assert oracle.mapreduce("identity", "affine", "f32", np.zeros((0, 2), np.float32)).tolist() == [1.0, 0.0]
    assert oracle.mapreduce("identity", "mat2", "u32", np.zeros((0, 4), np.uint32)).tolist() == [1, 0, 0, 1]
    assert oracle.mapreduce("identity", "quat", "f32", np.zeros((0, 4), np.float32)).tolist() == [1.0, 0.0, 0.0, 0.0]
    ident = oracle.mapreduce("identity", "argmax", None, np.zeros(0, oracle.ARGMAX_DTYPE))
    assert (int(ident["v"]), int(ident["idx"]), int(ident["cnt"])) == (-2 ** 31, 2 ** 31 - 1, 0)
    one = np.array([(5, 3, 2)], dtype=oracle.ARGMAX_DTYPE)
    assert oracle.mapreduce("identity", "argmax", None, one) == one[0]


def test_argmax_struct_is_max_first_position_and_total_count():
    x = ks_inputs.whole("argmax", 200_000)
    x["v"] = np.random.default_rng(8).integers(0, 40, size=len(x))     # many ties
    x["cnt"] = np.random.default_rng(9).integers(0, 1 << 40, size=len(x))
    got = oracle.mapreduce("identity", "argmax", None, x)
    vmax = int(x["v"].max())
    assert int(got["v"]) == vmax
    assert int(got["idx"]) == int(np.flatnonzero(x["v"] == vmax)[0])   # idx = position in this workload
    assert int(got["cnt"]) == sum(int(c) for c in x["cnt"])


def test_affine_fold_composes_the_maps_in_order():
    x = ks_inputs.whole("affine", 5000)
    a, b = (float(v) for v in oracle.mapreduce("identity", "affine", "f32", x))
    for x0 in (0.0, 1.0, -2.5):
        y = x0
        for ai, bi in x:
            y = float(ai) * y + float(bi)               # apply map 0, then map 1, ...
        assert a * x0 + b == pytest.approx(y, rel=1e-9, abs=1e-9)
    # exact in rationals on a short input
    short = x[:40]
    fa, fb = Fraction(1), Fraction(0)
    for ai, bi in short:
        fa, fb = Fraction(float(ai)) * fa, Fraction(float(ai)) * fb + Fraction(float(bi))
    a, b = (float(v) for v in oracle.mapreduce("identity", "affine", "f32", short))
    assert a == pytest.approx(float(fa), rel=1e-13) and b == pytest.approx(float(fb), rel=1e-12, abs=1e-13)


def test_mat2_fold_is_the_ordered_product_in_big_integers():
    m = ks_inputs.random_mat2(12, seed=11) | np.uint32(1)    # odd entries: the product does not collapse to zero
    p = [1, 0, 0, 1]
    for a, b, c, d in m.tolist():
        p = [p[0] * a + p[1] * c, p[0] * b + p[1] * d, p[2] * a + p[3] * c, p[2] * b + p[3] * d]
    assert oracle.mapreduce("identity", "mat2", "u32", m).tolist() == [v % (1 << 32) for v in p]
    # order matters: the reversed sequence gives another product
    assert oracle.mapreduce("identity", "mat2", "u32", m[::-1]).tolist() != [v % (1 << 32) for v in p]


def test_quaternion_fold_adds_rotation_angles_about_one_axis():
    angles = np.random.default_rng(12).uniform(-0.3, 0.3, size=500)
    axis = np.array([1.0, 2.0, -2.0]) / 3.0
    q = np.concatenate([np.cos(angles / 2)[:, None], np.sin(angles / 2)[:, None] * axis[None, :]], axis=1).astype(np.float32)
    got = oracle.mapreduce("identity", "quat", "f32", q)
    total = float(np.sum(2 * np.arctan2(np.linalg.norm(q[:, 1:].astype(np.float64), axis=1), q[:, 0].astype(np.float64))
                         * np.sign(angles)))
    want = np.concatenate([[math.cos(total / 2)], math.sin(total / 2) * axis])
    assert np.allclose(got, want, atol=1e-5)


def _all_parenthesisations(op, xs):
    if len(xs) == 1:
        return [xs[0]]
    out = []
    for k in range(1, len(xs)):
        for l in _all_parenthesisations(op, xs[:k]):
            for r in _all_parenthesisations(op, xs[k:]):
                out.append(op(l, r))
    return out


def test_every_order_and_grouping_on_tiny_inputs():
    rng = np.random.default_rng(13)
    # commutative operators: any order of the elements, any grouping, one answer (the paper's premise for mapreduce)
    for dt in ("i32", "u64"):
        x = rng.integers(np.iinfo(NP[dt]).min, np.iinfo(NP[dt]).max, size=6, dtype=NP[dt], endpoint=True)
        for op, py in (("sum", lambda l, r: wrap(l + r, dt)), ("min", min), ("max", max)):
            want = int(oracle.mapreduce("identity", op, dt, x))
            for perm in itertools.permutations([int(v) for v in x]):
                acc = perm[0]
                for v in perm[1:]:
                    acc = py(acc, v)
                assert acc == want
            assert set(_all_parenthesisations(py, [int(v) for v in x])) == {want}

    def argmax_op(l, r):
        take_r = r[0] > l[0] or (r[0] == l[0] and r[1] < l[1])
        return (r[0], r[1], l[2] + r[2]) if take_r else (l[0], l[1], l[2] + r[2])
    s = np.zeros(6, oracle.ARGMAX_DTYPE)
    s["v"], s["idx"], s["cnt"] = [3, 7, 7, 1, 7, 3], [10, 4, 2, 0, 9, 1], [1, 2, 3, 4, 5, 6]
    got = oracle.mapreduce("identity", "argmax", None, s)
    want = (int(got["v"]), int(got["idx"]), int(got["cnt"]))
    assert want == (7, 2, 21)
    for perm in itertools.permutations([tuple(int(v) for v in e) for e in s]):
        acc = perm[0]
        for v in perm[1:]:
            acc = argmax_op(acc, v)
        assert acc == want

    # non-commutative: every grouping that keeps the order equals the left fold; another order does not
    def mat_op(l, r):
        m = (1 << 32) - 1
        return ((l[0] * r[0] + l[1] * r[2]) & m, (l[0] * r[1] + l[1] * r[3]) & m,
                (l[2] * r[0] + l[3] * r[2]) & m, (l[2] * r[1] + l[3] * r[3]) & m)
    mats = ks_inputs.random_mat2(6, seed=14)
    want = tuple(oracle.mapreduce("identity", "mat2", "u32", mats).tolist())
    assert set(_all_parenthesisations(mat_op, [tuple(r) for r in mats.tolist()])) == {want}
    swapped = mats.copy()
    swapped[[0, 1]] = swapped[[1, 0]]
    assert tuple(oracle.mapreduce("identity", "mat2", "u32", swapped).tolist()) != want


# ---- bytes: the 8-bit types of the paper's mapreduce benchmark (Sec. VII-B, Tables I and III) ----

def _nearest_float32(fr: Fraction) -> np.float32:
    guess = np.float32(float(fr))
    around = (np.nextafter(guess, np.float32(-4)), guess, np.nextafter(guess, np.float32(4)))
    return min(around, key=lambda c: abs(Fraction(float(c)) - fr))


def test_unit_float8_levels_code_by_code():
    codes = np.arange(256, dtype=np.uint8)
    levels = oracle.apply_map("unit_float8", codes)
    assert levels.dtype == np.float32
    # 256 evenly spaced levels from -1 to +1: the end points, the order and the spacing fix the formula
    assert levels[0] == -1.0 and levels[255] == 1.0
    assert np.all(np.diff(levels.astype(np.float64)) > 0)
    assert np.abs(np.diff(levels.astype(np.float64)) - 2.0 / 255.0).max() <= 2.0 ** -24
    assert np.array_equal(levels, -levels[::-1])          # level(c) = -level(255 - c); no level is zero
    # promoted to float32 = the float32 NEAREST to the rational level, for every one of the 256 codes
    for c in range(256):
        assert levels[c] == _nearest_float32(Fraction(2 * c - 255, 255)), c
    with pytest.raises(TypeError):
        oracle.apply_map("unit_float8", np.zeros(4, np.int32))


def test_unit_float8_sum_closed_forms_and_exact_sum():
    codes = np.arange(256, dtype=np.uint8)
    # every level once: the levels cancel in pairs, and float64 holds every partial sum exactly
    assert float(oracle.mapreduce("unit_float8", "sum", "u8", codes)) == 0.0
    assert float(oracle.mapreduce("unit_float8", "sum", "u8", np.tile(codes, 1000))) == 0.0
    # n copies of one code: n times its float32 level, exact in float64
    n = 100_001
    for c in (0, 255, 128, 37):
        level = float(oracle.apply_map("unit_float8", np.array([c], np.uint8))[0])
        assert float(oracle.mapreduce("unit_float8", "sum", "u8", np.full(n, c, np.uint8))) == n * level
    x = np.random.default_rng(21).integers(0, 256, size=300_007, dtype=np.uint8)
    exact = math.fsum(float(_nearest_float32(Fraction(2 * c - 255, 255))) * k for c, k in enumerate(np.bincount(x, minlength=256)))
    assert abs(float(oracle.mapreduce("unit_float8", "sum", "u8", x)) - exact) <= 1e-9
    assert float(oracle.mapreduce("unit_float8", "sum", "u8", x, chunk=999)) == float(oracle.mapreduce("unit_float8", "sum", "u8", x))
    # the sign of the result is what the paper validates against a float64 reference
    assert float(oracle.mapreduce("unit_float8", "sum", "u8", np.full(7, 127, np.uint8))) < 0 < \
        float(oracle.mapreduce("unit_float8", "sum", "u8", np.full(7, 128, np.uint8)))
    assert float(oracle.mapreduce("unit_float8", "sum", "u8", x[:0])) == 0.0


def test_byte_sums_wide_and_in_the_element_type():
    x = np.random.default_rng(22).integers(0, 256, size=400_003, dtype=np.uint8)
    exact = sum(int(v) for v in x)
    assert int(oracle.mapreduce("widen64", "sum", "u8", x)) == exact == int(x.sum(dtype=np.uint64))
    assert oracle.mapreduce("widen64", "sum", "u8", x).dtype == np.uint64
    full = np.full(1 << 25, 255, np.uint8)                 # 255 * 2^25 > 2^32: a 32-bit sum would have wrapped
    assert int(oracle.mapreduce("widen64", "sum", "u8", full)) == 255 << 25
    # no map: UInt8 + UInt8 stays UInt8, so the sum is the exact sum modulo 2^8; numpy's own uint8 reduction agrees
    got = oracle.mapreduce("identity", "sum", "u8", x)
    assert got.dtype == np.uint8 and int(got) == exact % 256 == int(np.add.reduce(x, dtype=np.uint8))
    assert int(oracle.mapreduce("identity", "sum", "u8", x, chunk=1234)) == exact % 256
    assert int(oracle.mapreduce("identity", "sum", "u8", x[:0])) == 0 and int(oracle.mapreduce("widen64", "sum", "u8", x[:0])) == 0
    with pytest.raises(KeyError):
        oracle.mapreduce("identity", "max", "u8", x)


# ---- 16-bit floats, reduced after promotion to float32 ----

def _value_from_fields(bits: int, exp_bits: int, man_bits: int) -> float:
    """sign, exponent and mantissa fields -> value, written out from the IEEE definition (finite codes only)."""
    sign = -1.0 if bits >> (exp_bits + man_bits) else 1.0
    e = (bits >> man_bits) & ((1 << exp_bits) - 1)
    m = bits & ((1 << man_bits) - 1)
    bias = (1 << (exp_bits - 1)) - 1
    if e == 0:
        return sign * m * 2.0 ** (1 - bias - man_bits)
    return sign * (1.0 + m * 2.0 ** -man_bits) * 2.0 ** (e - bias)


@pytest.mark.parametrize("kind,exp_bits,man_bits", [("bf16", 8, 7), ("f16", 5, 10)])
def test_sixteen_bit_floats_promote_to_the_same_value(kind, exp_bits, man_bits):
    codes = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    values = oracle.apply_map("widen_f32", codes, kind)
    assert values.dtype == np.float32
    top = (1 << exp_bits) - 1
    finite = ((codes.astype(np.uint32) >> man_bits) & top) != top
    want = np.array([_value_from_fields(int(c), exp_bits, man_bits) for c in codes[finite]])
    assert np.array_equal(values[finite].astype(np.float64), want)          # every finite code, exactly
    assert np.all(~np.isfinite(values[~finite]))                            # the rest are infinities and NaNs
    assert float(values[0]) == 0.0 and np.signbit(values[0x8000])
    with pytest.raises(TypeError):
        oracle.apply_map("widen_f32", codes, None)
    with pytest.raises(TypeError):
        oracle.apply_map("widen_f32", codes.astype(np.int32), kind)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_sixteen_bit_float_reductions(kind):
    x = ks_inputs.random_half_bits(kind, 200_003, seed=23)
    values = oracle.apply_map("widen_f32", x, kind).astype(np.float64)
    exact = math.fsum(values)
    got = float(oracle.mapreduce("widen_f32", "sum", kind, x))
    assert abs(got - exact) <= len(x) * 2.0 ** -53 * max(1.0, np.abs(np.cumsum(values)).max())
    assert float(oracle.mapreduce("widen_f32", "max", kind, x)) == values.max()
    assert float(oracle.mapreduce("widen_f32", "min", kind, x)) == values.min()
    assert float(oracle.mapreduce("widen_f32", "sum", kind, x, chunk=4321)) == got
    one = {"bf16": 0x3F80, "f16": 0x3C00}[kind]
    n = 70_001
    assert float(oracle.mapreduce("widen_f32", "sum", kind, np.full(n, one, np.uint16))) == float(n)   # n ones
    assert float(oracle.mapreduce("widen_f32", "sum", kind, x[:0])) == 0.0
    assert float(oracle.mapreduce("widen_f32", "max", kind, x[:0])) == -np.inf
    with pytest.raises(KeyError):
        oracle.mapreduce("identity", "sum", kind, x)
