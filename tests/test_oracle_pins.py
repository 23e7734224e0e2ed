"""Pins for the CPU oracle (no GPU, no HIP library).

Each test fixes the oracle to something other than itself: a closed form, a
numpy / math library routine on a special case, an exact rational or integer
computation, a product worked out by hand, or brute force over every
parenthesisation of a tiny input.  Definition under test: paper Sec. II-C
(scan: out[i] = in[0] op ... op in[i], op associative, not necessarily
commutative) and Sec. V-B (inclusive or exclusive).
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import ks_inputs
import oracle

INT_TYPES = ["i32", "u32", "i64", "u64"]
BITS = {"i32": 32, "u32": 32, "i64": 64, "u64": 64}
NP = {"i32": np.int32, "u32": np.uint32, "i64": np.int64, "u64": np.uint64,
      "f32": np.float32, "f64": np.float64}


def wrap(value: int, dt: str) -> int:
    """Python integer -> the value a two's-complement / modular register would hold."""
    bits = BITS[dt]
    value &= (1 << bits) - 1
    if dt.startswith("i") and value >= 1 << (bits - 1):
        value -= 1 << bits
    return value


# ------------------------------------------------------------------ closed forms

@pytest.mark.parametrize("dt", INT_TYPES + ["f32", "f64"])
def test_all_ones_gives_1_to_n(dt):
    n = 100_000
    out = oracle.scan("sum", dt, np.ones(n, dtype=NP[dt]), inclusive=True)
    assert np.array_equal(out, np.arange(1, n + 1).astype(out.dtype))
    ex = oracle.scan("sum", dt, np.ones(n, dtype=NP[dt]), inclusive=False)
    assert np.array_equal(ex, np.arange(0, n).astype(ex.dtype))


def test_all_ones_f32_past_2_pow_24_is_still_exact_because_oracle_is_fp64():
    # a float32 accumulator would stall at 2^24; the oracle folds in double
    n = (1 << 24) + 1000
    out = oracle.scan("sum", "f32", np.ones(n, dtype=np.float32))
    assert out.dtype == np.float64
    assert out[-1] == float(n) and out[(1 << 24) + 5] == float((1 << 24) + 6)


@pytest.mark.parametrize("dt", INT_TYPES)
def test_iota_gives_triangular_numbers_mod_2w(dt):
    n = 200_000          # i(i+1)/2 passes 2^32 near i = 92682: the 32-bit types wrap
    x = np.arange(n, dtype=np.uint64).astype(NP[dt])
    out = oracle.scan("sum", dt, x)
    for i in [0, 1, 2, 65535, 65536, 92681, 92682, 131071, n - 1]:
        assert int(out[i]) == wrap(i * (i + 1) // 2, dt), i
    idx = np.arange(n, dtype=object)
    expect = [wrap(int(v), dt) for v in idx * (idx + 1) // 2]
    assert [int(v) for v in out] == expect


def test_iota_f64_triangular_exact():
    n = 100_000
    out = oracle.scan("sum", "f64", np.arange(n, dtype=np.float64))
    i = np.arange(n, dtype=np.float64)
    assert np.array_equal(out, i * (i + 1) / 2)


@pytest.mark.parametrize("dt", INT_TYPES)
def test_wraparound_is_modular(dt):
    info = np.iinfo(NP[dt])
    x = np.full(1000, info.max, dtype=NP[dt])
    out = oracle.scan("sum", dt, x)
    for i in [0, 1, 2, 3, 500, 999]:
        assert int(out[i]) == wrap((i + 1) * int(info.max), dt)
    ex = oracle.scan("sum", dt, x, inclusive=False)
    assert int(ex[0]) == 0 and int(ex[3]) == wrap(3 * int(info.max), dt)


# ------------------------------------------------------------------ library special cases

@pytest.mark.parametrize("dt", INT_TYPES)
def test_integer_sum_equals_numpy_cumsum(dt):
    rng = np.random.default_rng(11)
    info = np.iinfo(NP[dt])
    x = rng.integers(info.min, info.max, size=50_001, dtype=NP[dt], endpoint=True)
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.scan("sum", dt, x), np.cumsum(x, dtype=NP[dt]))


@pytest.mark.parametrize("dt", INT_TYPES + ["f32", "f64"])
def test_min_max_equal_numpy_accumulate(dt):
    rng = np.random.default_rng(12)
    if dt in BITS:
        info = np.iinfo(NP[dt])
        x = rng.integers(info.min, info.max, size=30_000, dtype=NP[dt], endpoint=True)
        lo, hi = info.min, info.max
    else:
        x = rng.normal(size=30_000).astype(NP[dt])
        lo, hi = -np.inf, np.inf
    assert np.array_equal(oracle.scan("max", dt, x), np.maximum.accumulate(x))
    assert np.array_equal(oracle.scan("min", dt, x), np.minimum.accumulate(x))
    exmax = oracle.scan("max", dt, x, inclusive=False)
    exmin = oracle.scan("min", dt, x, inclusive=False)
    assert exmax[0] == lo and exmin[0] == hi
    assert np.array_equal(exmax[1:], np.maximum.accumulate(x)[:-1])
    assert np.array_equal(exmin[1:], np.minimum.accumulate(x)[:-1])


def test_f32_sum_is_numpy_float64_cumsum():
    x = ks_inputs.whole("f32_sum", 300_000)
    assert np.array_equal(oracle.scan("sum", "f32", x), np.cumsum(x, dtype=np.float64))


@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_float_sum_against_exact_prefix_sums(dt):
    # math.fsum returns the correctly rounded exact sum of each prefix.
    rng = np.random.default_rng(13)
    x = (rng.random(3000) * 10.0 ** rng.integers(-6, 6, size=3000)).astype(NP[dt])
    x *= rng.choice([-1.0, 1.0], size=3000)
    out = oracle.scan("sum", dt, x)
    xs = [float(v) for v in x]
    scale = 0.0
    for i in range(len(xs)):
        exact = math.fsum(xs[: i + 1])
        scale += abs(xs[i])
        # a double left fold is within (i+1) * 2^-53 * sum|x| of the exact sum
        assert abs(out[i] - exact) <= (i + 1) * 2.0 ** -53 * scale + 5e-324


# ------------------------------------------------------------------ inclusive / exclusive, chunking

ALL_KINDS = [("sum", "i32"), ("sum", "u64"), ("sum", "f32"), ("sum", "f64"), ("max", "i64"),
             ("min", "f32"), ("affine", "f32"), ("argmax", None), ("mat2", "u32"), ("quat", "f32")]


def _sample(op, dt, n, seed):
    rng = np.random.default_rng(seed)
    if op == "affine":
        return ks_inputs.whole("affine", n, seed)
    if op == "argmax":
        return ks_inputs.whole("argmax", n, seed)
    if op == "mat2":
        return ks_inputs.random_mat2(n, seed)
    if op == "quat":
        return ks_inputs.random_unit_quats(n, seed)
    if dt in BITS:
        return rng.integers(-1000 if dt[0] == "i" else 0, 1000, size=n).astype(NP[dt])
    return rng.normal(size=n).astype(NP[dt])


@pytest.mark.parametrize("op,dt", ALL_KINDS)
def test_exclusive_is_inclusive_shifted_with_identity_in_front(op, dt):
    x = _sample(op, dt, 5000, 21)
    inc = oracle.scan(op, dt, x, True)
    exc = oracle.scan(op, dt, x, False)
    assert np.array_equal(exc[1:], inc[:-1])
    identity = {
        ("sum", dt): 0, ("max", "i64"): np.iinfo(np.int64).min, ("min", "f32"): np.inf,
        ("affine", "f32"): [1.0, 0.0], ("mat2", "u32"): [1, 0, 0, 1], ("quat", "f32"): [1.0, 0, 0, 0],
    }.get((op, dt))
    if op == "argmax":
        assert tuple(exc[0]) == (np.iinfo(np.int32).min, np.iinfo(np.int32).max, 0)
    else:
        assert np.array_equal(np.atleast_1d(exc[0]), np.atleast_1d(np.array(identity, dtype=exc.dtype)))


@pytest.mark.parametrize("op,dt", ALL_KINDS)
@pytest.mark.parametrize("inclusive", [True, False])
def test_streaming_in_chunks_equals_one_shot(op, dt, inclusive):
    x = _sample(op, dt, 4099, 22)
    whole = oracle.scan(op, dt, x, inclusive)
    for sizes in ([1, 1, 62, 1, 4034], [4099], [1000, 0, 3099], [63, 64, 65, 3907]):
        s = oracle.ScanStream(op, dt, inclusive)
        parts, at = [], 0
        for m in sizes:
            parts.append(s.feed(x[at:at + m]))
            at += m
        assert at == len(x)
        got = np.concatenate(parts)
        assert got.tobytes() == whole.tobytes()


def test_empty_input():
    for op, dt in ALL_KINDS:
        x = _sample(op, dt, 0, 1)
        assert oracle.scan(op, dt, x).shape[0] == 0


# ------------------------------------------------------------------ affine maps

def test_affine_hand_worked_order():
    # x -> 2x+1 then x -> 3x+4 is x -> 3(2x+1)+4 = 6x+7; the other order gives 2(3x+4)+1 = 6x+9.
    x = np.array([[2, 1], [3, 4]], dtype=np.float32)
    assert oracle.scan("affine", "f32", x)[1].tolist() == [6.0, 7.0]
    assert oracle.scan("affine", "f32", x[::-1].copy())[1].tolist() == [6.0, 9.0]
    # three maps: then x -> -x+0.5 : -(6x+7)+0.5 = -6x-6.5
    y = np.array([[2, 1], [3, 4], [-1, 0.5]], dtype=np.float32)
    assert oracle.scan("affine", "f32", y)[2].tolist() == [-6.0, -6.5]
    assert oracle.scan("affine", "f32", y, inclusive=False).tolist() == [[1, 0], [2, 1], [6, 7]]


def test_affine_constant_map_is_geometric_series():
    # (a,b) repeated: A_i = a^(i+1), B_i = b (a^(i+1) - 1)/(a - 1); exact in rationals.
    a, b, n = Fraction(3, 2), Fraction(-5, 4), 40
    x = np.tile(np.array([[float(a), float(b)]], dtype=np.float32), (n, 1))
    out = oracle.scan("affine", "f32", x)
    for i in range(n):
        A = a ** (i + 1)
        B = b * (A - 1) / (a - 1)
        assert out[i, 0] == pytest.approx(float(A), rel=1e-14)
        assert out[i, 1] == pytest.approx(float(B), rel=1e-13)


def test_affine_with_unit_slope_is_plain_sum_of_b():
    rng = np.random.default_rng(31)
    b = rng.uniform(-1, 1, 10_000).astype(np.float32)
    x = np.stack([np.ones_like(b), b], axis=1)
    out = oracle.scan("affine", "f32", x)
    assert np.array_equal(out[:, 0], np.ones(len(b)))
    assert np.array_equal(out[:, 1], np.cumsum(b, dtype=np.float64))


def test_affine_scan_solves_the_linear_recurrence():
    # x_i = a_i x_{i-1} + b_i from any x_0 equals A_i x_0 + B_i.
    x = ks_inputs.whole("affine", 20_000)
    out = oracle.scan("affine", "f32", x)
    for x0 in (0.0, 1.0, -3.25):
        v = x0
        for i in range(len(x)):
            v = float(x[i, 0]) * v + float(x[i, 1])
            if i % 997 == 0 or i == len(x) - 1:
                assert out[i, 0] * x0 + out[i, 1] == pytest.approx(v, rel=1e-9, abs=1e-9)


def test_affine_exact_against_rationals():
    rng = np.random.default_rng(32)
    a = rng.integers(-3, 4, size=25).astype(np.float32) / 2
    b = rng.integers(-8, 9, size=25).astype(np.float32) / 4
    out = oracle.scan("affine", "f32", np.stack([a, b], axis=1))
    A, B = Fraction(1), Fraction(0)
    for i in range(25):
        ra, rb = Fraction(float(a[i])), Fraction(float(b[i]))
        A, B = ra * A, ra * B + rb       # apply the accumulated map first, then the new one
        assert Fraction(out[i, 0]) == A and Fraction(out[i, 1]) == B   # dyadic, fits a double exactly


# ------------------------------------------------------------------ arg-max with count

def test_argmax_hand_worked_ties_keep_lowest_index():
    v = [5, 7, 7, 3, 9, 9, 1]
    x = np.array([(val, i, 1) for i, val in enumerate(v)], dtype=oracle.ARGMAX_DTYPE)
    out = oracle.scan("argmax", None, x)
    assert out["v"].tolist() == [5, 7, 7, 7, 9, 9, 9]
    assert out["idx"].tolist() == [0, 1, 1, 1, 4, 4, 4]
    assert out["cnt"].tolist() == [1, 2, 3, 4, 5, 6, 7]
    # lower index wins a tie even when it arrives later (operator property, not input order)
    y = np.array([(7, 10, 1), (7, 2, 5)], dtype=oracle.ARGMAX_DTYPE)
    assert tuple(oracle.scan("argmax", None, y)[1]) == (7, 2, 6)


def test_argmax_invariants_on_the_workload():
    x = ks_inputs.whole("argmax", 100_000)
    out = oracle.scan("argmax", None, x)
    v = x["v"]
    assert np.array_equal(out["cnt"], np.arange(1, len(x) + 1))
    assert np.array_equal(out["v"], np.maximum.accumulate(v))
    assert np.all(np.diff(out["idx"]) >= 0)
    assert np.array_equal(v[out["idx"]], out["v"])
    # idx is the FIRST position holding the running maximum
    first = np.zeros(len(v), dtype=np.int64)
    best, where = -1, -1
    for i, val in enumerate(v.tolist()):
        if val > best:
            best, where = val, i
        first[i] = where
    assert np.array_equal(out["idx"], first)


def test_argmax_count_wraps_and_extremes():
    x = np.array([(-2**31, 5, 2**63 - 1), (-2**31, 4, 1), (2**31 - 1, 9, 0)], dtype=oracle.ARGMAX_DTYPE)
    out = oracle.scan("argmax", None, x)
    assert tuple(out[1]) == (-2**31, 4, -2**63)
    assert tuple(out[2]) == (2**31 - 1, 9, -2**63)


# ------------------------------------------------------------------ 2x2 matrices mod 2^32

def test_mat2_hand_worked_order():
    # A = [[1,1],[0,1]], B = [[1,0],[1,1]]: AB = [[2,1],[1,1]], BA = [[1,1],[1,2]]
    A, B = [1, 1, 0, 1], [1, 0, 1, 1]
    assert oracle.scan("mat2", "u32", np.array([A, B], dtype=np.uint32))[1].tolist() == [2, 1, 1, 1]
    assert oracle.scan("mat2", "u32", np.array([B, A], dtype=np.uint32))[1].tolist() == [1, 1, 1, 2]


def test_mat2_fibonacci_closed_form_mod_2_32():
    # [[1,1],[1,0]]^k = [[F(k+1), F(k)], [F(k), F(k-1)]]
    n = 300
    x = np.tile(np.array([[1, 1, 1, 0]], dtype=np.uint32), (n, 1))
    out = oracle.scan("mat2", "u32", x)
    fib = [0, 1]
    while len(fib) < n + 2:
        fib.append(fib[-1] + fib[-2])
    for k in range(1, n + 1):
        expect = [fib[k + 1], fib[k], fib[k], fib[k - 1]]
        assert out[k - 1].tolist() == [e % (1 << 32) for e in expect]


def test_mat2_against_python_big_integers():
    x = ks_inputs.random_mat2(200, 41)
    out = oracle.scan("mat2", "u32", x)
    acc = None
    for i in range(len(x)):
        m = [[int(x[i, 0]), int(x[i, 1])], [int(x[i, 2]), int(x[i, 3])]]
        if acc is None:
            acc = m
        else:   # ordinary row-by-column product, accumulated matrix on the left
            acc = [[sum(acc[r][k] * m[k][c] for k in range(2)) % (1 << 32) for c in range(2)]
                   for r in range(2)]
        assert out[i].tolist() == [acc[0][0], acc[0][1], acc[1][0], acc[1][1]]


# ------------------------------------------------------------------ quaternions

def test_quat_units_do_not_commute():
    i, j = [0, 1, 0, 0], [0, 0, 1, 0]
    assert oracle.scan("quat", "f32", np.array([i, j], dtype=np.float32))[1].tolist() == [0, 0, 0, 1]    # ij = k
    assert oracle.scan("quat", "f32", np.array([j, i], dtype=np.float32))[1].tolist() == [0, 0, 0, -1]   # ji = -k
    assert oracle.scan("quat", "f32", np.array([i, i], dtype=np.float32))[1].tolist() == [-1, 0, 0, 0]   # i^2 = -1


def test_quat_same_axis_rotations_add_their_angles():
    axis = np.array([2.0, -1.0, 0.5]); axis /= np.linalg.norm(axis)
    theta, n = 0.01, 500
    q = np.concatenate([[math.cos(theta / 2)], math.sin(theta / 2) * axis]).astype(np.float32)
    # use the float32-rounded quaternion's own angle/axis for the closed form
    qd = q.astype(np.float64)
    norm = np.linalg.norm(qd)
    half = math.atan2(np.linalg.norm(qd[1:]), qd[0])
    ax = qd[1:] / np.linalg.norm(qd[1:])
    out = oracle.scan("quat", "f32", np.tile(q, (n, 1)))
    for k in (1, 2, 17, 250, 500):
        expect = norm ** k * np.concatenate([[math.cos(k * half)], math.sin(k * half) * ax])
        assert np.allclose(out[k - 1], expect, rtol=0, atol=1e-12)


def test_quat_matches_rotation_matrices():
    # the product of unit quaternions corresponds to the product of their rotation matrices
    def rot(q):
        w, x, y, z = q
        return np.array([[1 - 2 * (y * y + z * z), 2 * (x * y - z * w), 2 * (x * z + y * w)],
                         [2 * (x * y + z * w), 1 - 2 * (x * x + z * z), 2 * (y * z - x * w)],
                         [2 * (x * z - y * w), 2 * (y * z + x * w), 1 - 2 * (x * x + y * y)]])
    x = ks_inputs.random_unit_quats(50, 42)
    out = oracle.scan("quat", "f32", x)
    R = np.eye(3)
    for i in range(len(x)):
        q = x[i].astype(np.float64)
        R = R @ rot(q / np.linalg.norm(q))
        got = out[i] / np.linalg.norm(out[i])
        assert np.allclose(rot(got), R, atol=1e-9)


# ------------------------------------------------------------------ brute force over parenthesisations

def _all_groupings(items, op):
    """Every value obtainable by fully parenthesising items[0] op ... op items[-1] in order."""
    if len(items) == 1:
        return [items[0]]
    out = []
    for cut in range(1, len(items)):
        for left in _all_groupings(items[:cut], op):
            for right in _all_groupings(items[cut:], op):
                out.append(op(left, right))
    return out


def _py_ops():
    m32 = (1 << 32) - 1

    def affine(l, r):
        return (r[0] * l[0], r[0] * l[1] + r[1])

    def argmax(l, r):
        take_r = r[0] > l[0] or (r[0] == l[0] and r[1] < l[1])
        return (r[0] if take_r else l[0], r[1] if take_r else l[1], l[2] + r[2])

    def mat2(l, r):
        return ((l[0] * r[0] + l[1] * r[2]) & m32, (l[0] * r[1] + l[1] * r[3]) & m32,
                (l[2] * r[0] + l[3] * r[2]) & m32, (l[2] * r[1] + l[3] * r[3]) & m32)

    return affine, argmax, mat2


def test_every_parenthesisation_equals_the_left_fold_tiny_n():
    affine, argmax, mat2 = _py_ops()
    rng = np.random.default_rng(51)
    n = 7   # Catalan(6) = 132 groupings for the last prefix
    # integer sum with wrap
    xi = rng.integers(-2**31, 2**31, size=n, dtype=np.int64).astype(np.int32)
    got = oracle.scan("sum", "i32", xi)
    for i in range(n):
        vals = {wrap(v, "i32") for v in _all_groupings([int(v) for v in xi[: i + 1]], lambda a, b: a + b)}
        assert vals == {int(got[i])}
    # affine maps with small dyadic coefficients: exact in binary floating point
    a = rng.integers(-3, 4, size=n) / 2.0
    b = rng.integers(-6, 7, size=n) / 4.0
    got = oracle.scan("affine", "f32", np.stack([a, b], axis=1).astype(np.float32))
    for i in range(n):
        vals = set(_all_groupings([(Fraction(a[k]), Fraction(b[k])) for k in range(i + 1)], affine))
        assert vals == {(Fraction(got[i, 0]), Fraction(got[i, 1]))}
    # arg-max struct with many ties
    x = np.array([(int(v), int(idx), int(c)) for v, idx, c in
                  zip(rng.integers(0, 3, n), rng.permutation(n), rng.integers(1, 5, n))],
                 dtype=oracle.ARGMAX_DTYPE)
    got = oracle.scan("argmax", None, x)
    for i in range(n):
        vals = set(_all_groupings([tuple(int(f) for f in e) for e in x[: i + 1]], argmax))
        assert vals == {tuple(int(f) for f in got[i])}
    # 2x2 matrices mod 2^32
    m = ks_inputs.random_mat2(n, 52)
    got = oracle.scan("mat2", "u32", m)
    for i in range(n):
        vals = set(_all_groupings([tuple(int(f) for f in e) for e in m[: i + 1]], mat2))
        assert vals == {tuple(int(f) for f in got[i])}


def test_flipping_the_operands_changes_the_answer_for_noncommutative_ops():
    affine, _, mat2 = _py_ops()
    m = ks_inputs.random_mat2(6, 53)
    got = oracle.scan("mat2", "u32", m)
    flipped = oracle.fold_scan(lambda l, r: mat2(r, l), [tuple(int(f) for f in e) for e in m])
    assert [tuple(int(f) for f in e) for e in got] != flipped
    assert tuple(int(f) for f in got[0]) == flipped[0]
    # folding with the operands flipped is folding the reversed input: x5 * ... * x0
    rev = oracle.scan("mat2", "u32", m[::-1].copy())
    assert tuple(int(f) for f in rev[-1]) == flipped[-1]


def test_python_fold_matches_c_oracle_on_generic_objects():
    # fold_scan is the same definition over Python objects; strings make order visible.
    assert oracle.fold_scan(lambda a, b: a + b, list("abcd")) == ["a", "ab", "abc", "abcd"]
    assert oracle.fold_scan(lambda a, b: a + b, list("abcd"), inclusive=False, identity="") == ["", "a", "ab", "abc"]
    x = ks_inputs.whole("int32_sum", 1000)
    assert oracle.fold_scan(lambda a, b: wrap(a + b, "i32"), [int(v) for v in x]) == oracle.scan("sum", "i32", x).tolist()


# ------------------------------------------------------------------ the inputs themselves

def test_input_recipe_is_stable_and_in_range():
    a = ks_inputs.whole("int32_sum", 1 << 12)
    assert a.dtype == np.int32 and a.min() >= -100 and a.max() <= 100
    assert np.array_equal(a, ks_inputs.whole("int32_sum", 1 << 12))
    f = ks_inputs.whole("f32_sum", 1 << 12)
    assert f.dtype == np.float32 and f.min() >= 0 and f.max() < 1
    u = ks_inputs.whole("u64_exsum", 1 << 12)
    assert u.dtype == np.uint64 and int(u.max()) < 1 << 32
    p = ks_inputs.whole("affine", 1 << 12)
    assert p.shape == (1 << 12, 2) and p[:, 0].min() >= 0.99 and p[:, 0].max() <= 1.01 and abs(p[:, 1]).max() <= 1
    s = ks_inputs.whole("argmax", 1 << 12)
    assert s.dtype.itemsize == 16 and np.array_equal(s["idx"], np.arange(1 << 12)) and np.all(s["cnt"] == 1)
    assert s["v"].min() >= 0 and s["v"].max() < 1 << 20
    # chunked generation: chunks() concatenated is whole()
    assert np.array_equal(np.concatenate(list(ks_inputs.chunks("f32_sum", 5000))), ks_inputs.whole("f32_sum", 5000))


# ---------------------------------------------------------------- map-fused scan, scan(f, op, src) (paper Sec. IV-A)

def test_mapped_scan_with_identity_map_is_the_plain_scan():
    x = np.random.default_rng(5).integers(-9, 9, size=1000, dtype=np.int32)
    assert np.array_equal(oracle.mapped_scan("identity", "sum", "i32", x), oracle.scan("sum", "i32", x))


def test_square_sum_closed_form_sum_of_squares():
    n = 5000
    x = np.arange(1, n + 1, dtype=np.int32)
    got = oracle.mapped_scan("square", "sum", "i32", x)
    want = np.array([(k * (k + 1) * (2 * k + 1) // 6) % (1 << 32) for k in range(1, n + 1)], dtype=np.uint64)
    assert np.array_equal(got.view(np.uint32).astype(np.uint64), want)      # wraps from k = 1861 on
    # float32 inputs: squares exact in float64, prefix sums exact while they stay below 2^53
    xf = np.arange(1, 2001, dtype=np.float32)
    gotf = oracle.mapped_scan("square", "sum", "f32", xf)
    assert gotf.dtype == np.float64
    assert gotf.tolist() == [float(k * (k + 1) * (2 * k + 1) // 6) for k in range(1, 2001)]
    # exclusive: shifted, zero in front
    ex = oracle.mapped_scan("square", "sum", "f32", xf, inclusive=False)
    assert ex[0] == 0.0 and np.array_equal(ex[1:], gotf[:-1])


def test_square_map_rounds_nothing_for_float32_inputs():
    x = np.random.default_rng(6).uniform(-3, 3, size=1000).astype(np.float32)
    y = oracle.apply_map("square", x)
    assert all(Fraction(float(a)) ** 2 == Fraction(float(b)) for a, b in zip(x[:200], y[:200]))


def test_abs_max_is_running_maximum_of_magnitudes():
    x = np.random.default_rng(7).normal(size=4000).astype(np.float32)
    got = oracle.mapped_scan("abs", "max", "f32", x)
    assert np.array_equal(got, np.maximum.accumulate(np.abs(x)))
    assert np.all(np.diff(got) >= 0) and np.all(got >= np.abs(x))
    xi = np.array([3, -7, 5, np.iinfo(np.int32).min, 9], dtype=np.int32)
    # |INT32_MIN| wraps to itself, which is below every other magnitude in a signed maximum
    assert oracle.mapped_scan("abs", "max", "i32", xi).tolist() == [3, 7, 7, 7, 9]


def test_nonzero_sum_numbers_the_kept_elements_of_a_compaction():
    rng = np.random.default_rng(8)
    x = (rng.integers(0, 3, size=3000) * rng.integers(-5, 6, size=3000)).astype(np.int32)
    excl = oracle.mapped_scan("nonzero", "sum", "i32", x, inclusive=False)
    incl = oracle.mapped_scan("nonzero", "sum", "i32", x, inclusive=True)
    kept = np.flatnonzero(x)
    assert np.array_equal(excl[kept], np.arange(len(kept), dtype=np.int32))   # position of each kept element
    assert incl[-1] == len(kept) and np.array_equal(incl, np.cumsum(x != 0).astype(np.int32))
    compacted = np.empty(len(kept), dtype=np.int32)
    compacted[excl[kept]] = x[kept]
    assert np.array_equal(compacted, x[x != 0])


# ---------------------------------------------------------------- element types wider than / not a power of two of 16 bytes

def test_mat2_u64_hand_product_fibonacci_and_big_integers():
    # hand-worked: [[1,2],[3,4]] * [[5,6],[7,8]] = [[19,22],[43,50]], and the other order differs
    a, b = [1, 2, 3, 4], [5, 6, 7, 8]
    x = np.array([a, b], dtype=np.uint64)
    assert oracle.scan("mat2", "u64", x)[1].tolist() == [19, 22, 43, 50]
    assert oracle.scan("mat2", "u64", x[::-1].copy())[1].tolist() == [23, 34, 31, 46]
    # Fibonacci closed form mod 2^64: [[1,1],[1,0]]^k = [[F(k+1), F(k)], [F(k), F(k-1)]]
    n = 500
    out = oracle.scan("mat2", "u64", np.tile(np.array([[1, 1, 1, 0]], dtype=np.uint64), (n, 1)))
    f0, f1, mask = 0, 1, (1 << 64) - 1
    for k in range(1, n + 1):
        f0, f1 = f1, f0 + f1                       # f0 = F(k), f1 = F(k+1), exact Python integers
        assert out[k - 1].tolist() == [f1 & mask, f0 & mask, f0 & mask, (f1 - f0) & mask]
    # random matrices against Python big integers, inclusive and exclusive
    m = ks_inputs.random_mat2_wide(200, seed=5)
    inc, exc = oracle.scan("mat2", "u64", m, True), oracle.scan("mat2", "u64", m, False)
    p = [1, 0, 0, 1]
    for i, (e, f, g, h) in enumerate(m.tolist()):
        assert exc[i].tolist() == [v & mask for v in p]
        p = [p[0] * e + p[1] * g, p[0] * f + p[1] * h, p[2] * e + p[3] * g, p[2] * f + p[3] * h]
        p = [v & mask for v in p]
        assert inc[i].tolist() == p
    # streamed in chunks = one shot
    s = oracle.ScanStream("mat2", "u64", True)
    assert np.array_equal(np.concatenate([s.feed(m[:77]), s.feed(m[77:])]), inc)


def test_range_with_count_is_running_min_max_and_count():
    x = ks_inputs.random_ranges(50_000, seed=6)
    assert x.dtype.itemsize == 12
    inc, exc = oracle.scan("range", None, x, True), oracle.scan("range", None, x, False)
    assert np.array_equal(inc["lo"], np.minimum.accumulate(x["lo"]))
    assert np.array_equal(inc["hi"], np.maximum.accumulate(x["hi"]))
    assert np.array_equal(inc["cnt"], np.cumsum(x["cnt"].astype(np.uint64)).astype(np.uint32))   # mod 2^32
    assert (int(exc[0]["lo"]), int(exc[0]["hi"]), int(exc[0]["cnt"])) == (2 ** 31 - 1, -2 ** 31, 0)
    assert np.array_equal(exc[1:], inc[:-1])
    # commutative and associative: every order of six elements folds to the same value
    import itertools
    six = x[:6]
    want = oracle.mapreduce("identity", "range", None, six)
    for perm in itertools.permutations(range(6)):
        assert oracle.mapreduce("identity", "range", None, six[list(perm)]) == want
