/*
 * TEST INFRASTRUCTURE -- sequential CPU oracle for the device-wide scan.
 *
 * This file is the reference the GPU library is checked against.  It is not
 * part of the product: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper
 * with the HIP sources, and it is deliberately the slowest obvious thing.
 *
 * What it computes (paper, Sec. II-C "Parallel primitives", scan; Sec. V-B
 * "Scan", first sentence): for an associative, not necessarily commutative
 * operator op,
 *
 *     inclusive:  out[i] = in[0] op in[1] op ... op in[i]
 *     exclusive:  out[i] = in[0] op ... op in[i-1],   out[0] = identity(op)
 *
 * The device algorithm reaches exactly this result (up to rounding order for
 * floating point), so the oracle is the definition written as one left fold:
 * the running value is always the LEFT operand, the new element the RIGHT.
 *
 * Readings where the paper is silent:
 *   - exclusive scans start from the operator's identity;
 *   - integer sums wrap (computed in unsigned arithmetic);
 *   - float32 inputs are folded in double and returned as double, float64
 *     inputs are folded in long double and returned as double.  min/max are
 *     exact in any order, so they are folded in the input type.
 *
 * Every routine is a stream: `state` carries the running value between calls
 * so that arrays larger than host memory can be fed in chunks.  state->started
 * is 0 before the first element of the whole sequence has been consumed.
 *
 * Pins (tests/test_oracle_pins.py): closed forms (all-ones, x_i = i, constant
 * affine map = geometric series), numpy cumsum / maximum.accumulate special
 * cases, math.fsum per-prefix exact sums, every parenthesisation on tiny n,
 * operand-order checks with non-commutative operators, the inclusive /
 * exclusive shift relation, chunk independence, and the affine <-> linear
 * recurrence equivalence.
 */
#include <stddef.h>
#include <stdint.h>

/* ------------------------------------------------------------------ */
/* scalar sum / min / max                                              */
/* ------------------------------------------------------------------ */

#define ORACLE_SCALAR_SCAN(NAME, IN_T, ACC_T, OUT_T, IDENTITY, COMBINE)          \
    typedef struct { ACC_T acc; int started; } NAME##_state;                      \
    void NAME(const IN_T *in, OUT_T *out, size_t n, int inclusive,                \
              NAME##_state *state)                                                \
    {                                                                             \
        for (size_t i = 0; i < n; ++i) {                                          \
            ACC_T x = (ACC_T)in[i];                                               \
            if (inclusive) {                                                      \
                ACC_T l = state->acc;                                             \
                state->acc = state->started ? (COMBINE) : x;                      \
                state->started = 1;                                               \
                out[i] = (OUT_T)state->acc;                                       \
            } else {                                                              \
                if (!state->started) { state->acc = (ACC_T)(IDENTITY); state->started = 1; } \
                out[i] = (OUT_T)state->acc;                                       \
                ACC_T l = state->acc;                                             \
                state->acc = (COMBINE);                                           \
            }                                                                     \
        }                                                                         \
    }

/* integer sums: unsigned accumulators give two's-complement wrap without UB */
ORACLE_SCALAR_SCAN(oracle_sum_i32, int32_t,  uint32_t, int32_t,  0u,   l + x)
ORACLE_SCALAR_SCAN(oracle_sum_u32, uint32_t, uint32_t, uint32_t, 0u,   l + x)
ORACLE_SCALAR_SCAN(oracle_sum_i64, int64_t,  uint64_t, int64_t,  0ull, l + x)
ORACLE_SCALAR_SCAN(oracle_sum_u64, uint64_t, uint64_t, uint64_t, 0ull, l + x)
/* floating sums: one precision step above the input */
ORACLE_SCALAR_SCAN(oracle_sum_f32, float,  double,      double, 0.0,  l + x)
ORACLE_SCALAR_SCAN(oracle_sum_f64, double, long double, double, 0.0L, l + x)

ORACLE_SCALAR_SCAN(oracle_max_i32, int32_t,  int32_t,  int32_t,  INT32_MIN,  (x > l ? x : l))
ORACLE_SCALAR_SCAN(oracle_max_u32, uint32_t, uint32_t, uint32_t, 0u,         (x > l ? x : l))
ORACLE_SCALAR_SCAN(oracle_max_i64, int64_t,  int64_t,  int64_t,  INT64_MIN,  (x > l ? x : l))
ORACLE_SCALAR_SCAN(oracle_max_u64, uint64_t, uint64_t, uint64_t, 0ull,       (x > l ? x : l))
ORACLE_SCALAR_SCAN(oracle_max_f32, float,    float,    float,    (-__builtin_inff()), (x > l ? x : l))
ORACLE_SCALAR_SCAN(oracle_max_f64, double,   double,   double,   (-__builtin_inf()),  (x > l ? x : l))

ORACLE_SCALAR_SCAN(oracle_min_i32, int32_t,  int32_t,  int32_t,  INT32_MAX,  (x < l ? x : l))
ORACLE_SCALAR_SCAN(oracle_min_u32, uint32_t, uint32_t, uint32_t, UINT32_MAX, (x < l ? x : l))
ORACLE_SCALAR_SCAN(oracle_min_i64, int64_t,  int64_t,  int64_t,  INT64_MAX,  (x < l ? x : l))
ORACLE_SCALAR_SCAN(oracle_min_u64, uint64_t, uint64_t, uint64_t, UINT64_MAX, (x < l ? x : l))
ORACLE_SCALAR_SCAN(oracle_min_f32, float,    float,    float,    (__builtin_inff()), (x < l ? x : l))
ORACLE_SCALAR_SCAN(oracle_min_f64, double,   double,   double,   (__builtin_inf()),  (x < l ? x : l))

/* ------------------------------------------------------------------ */
/* affine-map composition (non-commutative)                            */
/* ------------------------------------------------------------------ */
/*
 * Element (a, b) stands for the map x -> a*x + b.  L op R means "apply L
 * first, then R":  (R.a*L.a, R.a*L.b + R.b).  Identity (1, 0).  Inputs are
 * float32 pairs stored interleaved; folded and returned in double.
 */
typedef struct { double a, b; int started; } oracle_affine_state;

void oracle_affine_f32(const float *in, double *out, size_t n, int inclusive,
                       oracle_affine_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        double ra = (double)in[2 * i], rb = (double)in[2 * i + 1];
        if (!state->started) {
            state->started = 1;
            if (inclusive) { state->a = ra; state->b = rb; out[2 * i] = ra; out[2 * i + 1] = rb; continue; }
            state->a = 1.0; state->b = 0.0;
        }
        double la = state->a, lb = state->b;
        double na = ra * la;
        double nb = ra * lb + rb;
        if (inclusive) {
            out[2 * i] = na; out[2 * i + 1] = nb;
        } else {
            out[2 * i] = la; out[2 * i + 1] = lb;
        }
        state->a = na; state->b = nb;
    }
}

/* ------------------------------------------------------------------ */
/* running arg-max with count (16-byte integer struct)                 */
/* ------------------------------------------------------------------ */
/*
 * Element {v, idx, cnt}.  L op R keeps the larger v; on equal v the lower idx;
 * cnt adds (wrapping).  Identity {INT32_MIN, INT32_MAX, 0}.
 */
typedef struct { int32_t v; int32_t idx; int64_t cnt; } oracle_argmax_t;
typedef struct { oracle_argmax_t acc; int started; } oracle_argmax_state;

static oracle_argmax_t argmax_combine(oracle_argmax_t l, oracle_argmax_t r)
{
    oracle_argmax_t o;
    int take_r = (r.v > l.v) || (r.v == l.v && r.idx < l.idx);
    o.v = take_r ? r.v : l.v;
    o.idx = take_r ? r.idx : l.idx;
    o.cnt = (int64_t)((uint64_t)l.cnt + (uint64_t)r.cnt);
    return o;
}

void oracle_argmax(const oracle_argmax_t *in, oracle_argmax_t *out, size_t n,
                   int inclusive, oracle_argmax_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        if (!state->started) {
            state->started = 1;
            if (inclusive) { state->acc = in[i]; out[i] = in[i]; continue; }
            state->acc.v = INT32_MIN; state->acc.idx = INT32_MAX; state->acc.cnt = 0;
        }
        oracle_argmax_t next = argmax_combine(state->acc, in[i]);
        out[i] = inclusive ? next : state->acc;
        state->acc = next;
    }
}

/* ------------------------------------------------------------------ */
/* 2x2 matrix product over Z / 2^32 (non-commutative, exact)           */
/* ------------------------------------------------------------------ */
/*
 * Element = row-major {m00, m01, m10, m11}.  L op R = L * R (ordinary matrix
 * product, earlier element on the left), entries mod 2^32.  Identity = I.
 */
typedef struct { uint32_t m[4]; } oracle_mat2_t;
typedef struct { oracle_mat2_t acc; int started; } oracle_mat2_state;

static oracle_mat2_t mat2_mul(oracle_mat2_t l, oracle_mat2_t r)
{
    oracle_mat2_t o;
    o.m[0] = l.m[0] * r.m[0] + l.m[1] * r.m[2];
    o.m[1] = l.m[0] * r.m[1] + l.m[1] * r.m[3];
    o.m[2] = l.m[2] * r.m[0] + l.m[3] * r.m[2];
    o.m[3] = l.m[2] * r.m[1] + l.m[3] * r.m[3];
    return o;
}

void oracle_mat2_u32(const oracle_mat2_t *in, oracle_mat2_t *out, size_t n,
                     int inclusive, oracle_mat2_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        if (!state->started) {
            state->started = 1;
            if (inclusive) { state->acc = in[i]; out[i] = in[i]; continue; }
            state->acc.m[0] = 1; state->acc.m[1] = 0; state->acc.m[2] = 0; state->acc.m[3] = 1;
        }
        oracle_mat2_t next = mat2_mul(state->acc, in[i]);
        out[i] = inclusive ? next : state->acc;
        state->acc = next;
    }
}

/* ------------------------------------------------------------------ */
/* quaternion (Hamilton) product, float32 in, double out               */
/* ------------------------------------------------------------------ */
/*
 * Element = {w, x, y, z}.  L op R = Hamilton product L*R (the paper's example
 * of a non-commutative operator, Sec. V-B last paragraph).  Identity (1,0,0,0).
 */
typedef struct { double q[4]; int started; } oracle_quat_state;

void oracle_quat_f32(const float *in, double *out, size_t n, int inclusive,
                     oracle_quat_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        double rw = in[4 * i], rx = in[4 * i + 1], ry = in[4 * i + 2], rz = in[4 * i + 3];
        if (!state->started) {
            state->started = 1;
            if (inclusive) {
                state->q[0] = rw; state->q[1] = rx; state->q[2] = ry; state->q[3] = rz;
                for (int k = 0; k < 4; ++k) out[4 * i + k] = state->q[k];
                continue;
            }
            state->q[0] = 1.0; state->q[1] = 0.0; state->q[2] = 0.0; state->q[3] = 0.0;
        }
        double lw = state->q[0], lx = state->q[1], ly = state->q[2], lz = state->q[3];
        double nw = lw * rw - lx * rx - ly * ry - lz * rz;
        double nx = lw * rx + lx * rw + ly * rz - lz * ry;
        double ny = lw * ry - lx * rz + ly * rw + lz * rx;
        double nz = lw * rz + lx * ry - ly * rx + lz * rw;
        if (inclusive) {
            out[4 * i] = nw; out[4 * i + 1] = nx; out[4 * i + 2] = ny; out[4 * i + 3] = nz;
        } else {
            out[4 * i] = lw; out[4 * i + 1] = lx; out[4 * i + 2] = ly; out[4 * i + 3] = lz;
        }
        state->q[0] = nw; state->q[1] = nx; state->q[2] = ny; state->q[3] = nz;
    }
}

/* ------------------------------------------------------------------ */
/* 2x2 matrix product over Z / 2^64: a 32-byte element                 */
/* ------------------------------------------------------------------ */
/*
 * The same operator as above on 64-bit entries (paper Sec. IV-A: elements may
 * be any struct of plain fields, whatever their size).  Row-major {m00, m01,
 * m10, m11}; L op R = L * R, entries mod 2^64; identity = I.
 */
typedef struct { uint64_t m[4]; } oracle_mat2w_t;
typedef struct { oracle_mat2w_t acc; int started; } oracle_mat2w_state;

void oracle_mat2_u64(const oracle_mat2w_t *in, oracle_mat2w_t *out, size_t n,
                     int inclusive, oracle_mat2w_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        if (!state->started) {
            state->started = 1;
            if (inclusive) { state->acc = in[i]; out[i] = in[i]; continue; }
            state->acc.m[0] = 1; state->acc.m[1] = 0; state->acc.m[2] = 0; state->acc.m[3] = 1;
        }
        const oracle_mat2w_t l = state->acc, r = in[i];
        oracle_mat2w_t next;
        next.m[0] = l.m[0] * r.m[0] + l.m[1] * r.m[2];
        next.m[1] = l.m[0] * r.m[1] + l.m[1] * r.m[3];
        next.m[2] = l.m[2] * r.m[0] + l.m[3] * r.m[2];
        next.m[3] = l.m[2] * r.m[1] + l.m[3] * r.m[3];
        out[i] = inclusive ? next : state->acc;
        state->acc = next;
    }
}

/* ------------------------------------------------------------------ */
/* running range with count: a 12-byte element                         */
/* ------------------------------------------------------------------ */
/*
 * Element {lo, hi, cnt}: the smallest and the largest value seen and how many
 * (an input element is {x, x, 1}).  L op R = {min(L.lo, R.lo), max(L.hi, R.hi),
 * L.cnt + R.cnt mod 2^32}.  Identity {INT32_MAX, INT32_MIN, 0}.  Commutative.
 * Twelve bytes: a size that is not a power of two (paper Sec. IV-A).
 */
typedef struct { int32_t lo; int32_t hi; uint32_t cnt; } oracle_range_t;
typedef struct { oracle_range_t acc; int started; } oracle_range_state;

void oracle_range_i32(const oracle_range_t *in, oracle_range_t *out, size_t n,
                      int inclusive, oracle_range_state *state)
{
    for (size_t i = 0; i < n; ++i) {
        if (!state->started) {
            state->started = 1;
            if (inclusive) { state->acc = in[i]; out[i] = in[i]; continue; }
            state->acc.lo = INT32_MAX; state->acc.hi = INT32_MIN; state->acc.cnt = 0;
        }
        const oracle_range_t l = state->acc, r = in[i];
        oracle_range_t next;
        next.lo = r.lo < l.lo ? r.lo : l.lo;
        next.hi = r.hi > l.hi ? r.hi : l.hi;
        next.cnt = l.cnt + r.cnt;
        out[i] = inclusive ? next : state->acc;
        state->acc = next;
    }
}
