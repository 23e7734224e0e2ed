/*
 * ks_scan -- device-wide inclusive / exclusive scan for AMD MI355X (gfx950).
 *
 * C ABI of the library.  Operation defined in the paper, Sec. II-C (parallel
 * primitives: scan is dst[i] = src[0] op ... op src[i] for an associative, not
 * necessarily commutative op) and Sec. V-B (inclusive or exclusive prefix
 * reduction, single pass with decoupled look-back).  Every step of the path
 * runs in the library's own HIP kernels; there is no CPU fallback.
 *
 * General conventions
 *   - `in`, `out`, `temp` are DEVICE pointers owned by the caller.  `in` and
 *     `out` hold n contiguous elements of the given dtype and must be aligned
 *     to the element's alignment (4 or 8 bytes, see ks_dtype).  Nothing more
 *     is needed: every access is a range-checked 16-byte buffer instruction,
 *     so slices that start at any element run at the same speed.
 *   - Element sizes (paper Sec. IV-A: any struct of plain fields): 4, 8 and 16
 *     bytes run in every kernel shape; other sizes that divide 128 or 144 bytes
 *     (here 12 and 32) run in the one shape where a lane holds 8 or 9
 *     consecutive 16-byte granules, in both strategies, in ks_scan_strided and in
 *     ks_mapreduce; the shape options "waves" / "form" do not apply to them.
 *     One-byte elements (KS_U8) are reduced only (ks_mapreduce).
 *   - 16-bit floats (KS_BF16, KS_F16; KS_SUM, KS_MIN, KS_MAX): every element is
 *     promoted to float as it is loaded and the arithmetic is float's (sums: as
 *     for KS_F32); a scan rounds every output to the 16-bit type, to nearest, ties
 *     to even (sums beyond the type's range become infinities), so running minima
 *     and maxima are exact and a sum output lies within half a unit in the last
 *     place of the float result.  For the scans both arrays must start on a 4-byte
 *     boundary (n may be odd: what lies behind the output is not touched);
 *     ks_scan_strided does not take them.  ks_mapreduce takes them at any 2-byte
 *     address, with KS_MAP_WIDEN_F32, and writes a float.
 *   - in == out (exactly in place) is allowed; any other overlap is rejected.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise (except ks_scan_check)
 *     and never throw.  n == 0 returns KS_OK without a launch.
 *   - Return value: KS_OK (0) or a negative ks_status.
 *   - In an exclusive scan out[0] is the operator's identity; the accumulated
 *     (earlier) value is always the left operand of op.
 */
#ifndef KS_SCAN_H
#define KS_SCAN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KS_OK = 0,
    KS_ERR_INVALID_ARG = -1, /* null pointer with n > 0, bad enum value                      */
    KS_ERR_UNSUPPORTED = -2, /* (dtype, op) pair, (dtype, map, op) triple or forced kernel shape
                                that is not compiled                                         */
    KS_ERR_MISALIGNED = -3,  /* pointer not aligned to the element type                      */
    KS_ERR_OVERLAP = -4,     /* in and out overlap without being identical                   */
    KS_ERR_WORKSPACE = -5,   /* temp too small / misaligned, or internal allocation failed   */
    KS_ERR_HIP = -6,         /* a HIP call failed; raw code via ks_last_hip_error()          */
    KS_ERR_TIMEOUT = -7      /* a look-back wait hit its spin limit (see ks_scan_check)      */
} ks_status;

/* Element types.  Structs are plain little-endian C structs, naturally aligned. */
typedef enum {
    KS_I32 = 0,              /* int32_t                                              4 B */
    KS_U32 = 1,              /* uint32_t                                             4 B */
    KS_I64 = 2,              /* int64_t                                              8 B */
    KS_U64 = 3,              /* uint64_t                                             8 B */
    KS_F32 = 4,              /* float                                                4 B */
    KS_F64 = 5,              /* double                                               8 B */
    KS_AFFINE_F32 = 6,       /* struct { float a, b; }  the map x -> a*x + b         8 B */
    KS_ARGMAX_I32_CNT64 = 7, /* struct { int32_t v; int32_t idx; int64_t cnt; }     16 B */
    KS_MAT2_U32 = 8,         /* struct { uint32_t m00, m01, m10, m11; } row-major   16 B */
    KS_QUAT_F32 = 9,         /* struct { float w, x, y, z; }                        16 B */
    KS_MAT2_U64 = 10,        /* struct { uint64_t m00, m01, m10, m11; } row-major   32 B */
    KS_RANGE_I32_CNT32 = 11, /* struct { int32_t lo, hi; uint32_t cnt; }            12 B */
    KS_U8 = 12,              /* uint8_t; ks_mapreduce only (the scans refuse it)     1 B */
    KS_BF16 = 13,            /* bfloat16 as uint16_t bits (see "16-bit floats" below)  2 B */
    KS_F16 = 14,             /* IEEE binary16 as uint16_t bits                        2 B */
    KS_DTYPE_COUNT = 15
} ks_dtype;

/* Operators; L is the accumulated (earlier) operand, R the later one. */
typedef enum {
    KS_SUM = 0,            /* L + R (integers wrap); identity 0.  All six scalar types; KS_U8 in
                              ks_mapreduce                                                       */
    KS_MIN = 1,            /* min(L, R); identity = largest value (+inf).  Scalar types          */
    KS_MAX = 2,            /* max(L, R); identity = smallest value (-inf). Scalar types.  With NaN
                              among float inputs the results of min / max from that element on
                              are unspecified (the comparisons are evaluated in an order that
                              depends on the tiling); the sign of a zero result (a sum that comes
                              out as zero, a minimum or maximum over +0 and -0) is unspecified too */
    KS_AFFINE_COMPOSE = 3, /* apply L then R: (R.a*L.a, R.a*L.b + R.b); identity (1,0)           */
    KS_ARGMAX_COUNT = 4,   /* larger v wins, equal v: lower idx wins; cnt adds (wraps);
                              identity {INT32_MIN, INT32_MAX, 0}                                 */
    KS_MAT2_MUL = 5,       /* 2x2 matrix product L*R, entries mod 2^32 (KS_MAT2_U32) or 2^64
                              (KS_MAT2_U64); identity I                                          */
    KS_QUAT_MUL = 6,       /* Hamilton product L*R (paper Sec. V-B, non-commutative example);
                              identity (1,0,0,0)                                                 */
    KS_RANGE_COUNT = 7,    /* {min(L.lo, R.lo), max(L.hi, R.hi), L.cnt + R.cnt mod 2^32}; identity
                              {INT32_MAX, INT32_MIN, 0}                                          */
    KS_OP_COUNT = 8
} ks_op;

/* Cross-workgroup strategy. */
typedef enum {
    KS_ALGO_AUTO = 0,             /* library's choice for (dtype, n)                              */
    KS_ALGO_LOOKBACK = 1,         /* one kernel, decoupled look-back (paper Sec. V-B): 2n traffic  */
    KS_ALGO_REDUCE_THEN_SCAN = 2  /* three kernels per level, no inter-workgroup waiting,
                                     deterministic for floating point: 3n traffic                 */
} ks_algo;

/*
 * Element-wise maps for the map-fused scan and mapreduce (paper Sec. IV-A: the
 * high-level interface scan(f, op, src), mapreduce(f, op, src)).  The map is
 * applied as elements are loaded.  The first four are T -> T: the output has the
 * input's element type.  The others take KS_U8, KS_BF16 or KS_F16 and change the
 * type (f: T -> S of Sec. II-C); only ks_mapreduce accepts them, and its result is
 * an S.
 */
typedef enum {
    KS_MAP_IDENTITY = 0,
    KS_MAP_SQUARE = 1,      /* x * x (integers wrap)                                            */
    KS_MAP_ABS = 2,         /* |x| (the most negative integer maps to itself)                   */
    KS_MAP_NONZERO = 3,     /* x != 0 ? 1 : 0, e.g. sum scan = positions of a stream compaction */
    KS_MAP_UNIT_FLOAT8 = 4, /* uint8_t code c -> float: level c of 256 evenly spaced levels from
                               -1 to +1 (the 8-bit type of the paper's mapreduce benchmark,
                               Sec. VII-B), the float nearest to (2c - 255) / 255           */
    KS_MAP_WIDEN64 = 5,     /* uint8_t -> uint64_t, so that a sum of bytes cannot wrap          */
    KS_MAP_WIDEN_F32 = 6,   /* KS_BF16 / KS_F16 -> the float of the same value (exact)          */
    KS_MAP_COUNT = 7
} ks_map;

/*
 * Scan n elements of `in` into `out` on `stream` (paper Sec. V-B).
 * Uses a library-owned scratch buffer cached per (device, stream); the first
 * call on a stream, or a call that needs a larger one, allocates device memory.
 * Back-to-back calls on one stream are safe; calls on different streams use
 * different buffers.  inclusive: non-zero = inclusive, 0 = exclusive.
 * Under stream capture the call is recorded if the stream's scratch is already
 * large enough (make an eager call with at least the same n on that stream
 * first); otherwise it returns KS_ERR_WORKSPACE and records nothing.  A recorded
 * call clears its scratch with a kernel of its own on every replay, and a
 * scratch buffer that a graph has recorded is never freed.  Callers that must
 * not depend on any of this use ks_scan_with_temp.
 */
int ks_scan(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n,
            void *stream);

/*
 * Seeded scan: one piece of a longer sequence (paper Sec. II-C with everything
 * before in[0] already folded into one value):
 *     out[i] = seed op in[0] op ... op in[i]     (inclusive)
 *     out[i] = seed op in[0] op ... op in[i-1]   (exclusive; out[0] = seed)
 * `seed` is a device pointer to ONE element of dtype, read when the call runs on
 * the stream (it may be the last output of the call before, or lie inside `out`).
 * This is what scanning an array chunk by chunk, or shard by shard on several
 * devices, needs: the seed of a piece is the total of the pieces before it.  The
 * seed is the LEFT operand, so operators that do not commute are served; no map is
 * applied to it, and float sums carry it in double like every other prefix.
 * Always the single-pass algorithm with the library-owned scratch; one small
 * extra kernel stores the seed.  Other arguments, streams, graphs and errors as for
 * ks_scan; seed == NULL with n > 0 is KS_ERR_INVALID_ARG.
 */
int ks_scan_seeded(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n,
                   const void *seed, void *stream);

/*
 * Map-fused scan (paper Sec. IV-A, scan(f, op, src)):
 *     out[i] = f(in[0]) op f(in[1]) op ... op f(in[i])     (inclusive)
 * with f one of ks_map; arguments, workspace, stream behaviour and errors as for
 * ks_scan.  KS_MAP_IDENTITY is ks_scan.  Instantiated (dtype, map, op) triples:
 * see ks_map_supported; others return KS_ERR_UNSUPPORTED.  Mapped scans choose
 * their kernel shapes as the plain pair does (of the shape options, those within
 * what the defaults can select apply).
 */
int ks_scan_map(ks_dtype dtype, ks_map map, ks_op op, int inclusive, const void *in, void *out,
                size_t n, void *stream);

/*
 * Scan of strided views (paper Sec. IV-C, the element-wise fallback for data
 * that is not contiguous): element i of the input is in[i * in_stride], element
 * i of the output out[i * out_stride], strides in elements, >= 1 and <= 2^20
 * (e.g. one column of a row-major matrix).  Elements between the strides are
 * neither read nor written.  Runs the single-pass look-back scan (Sec. V-B) with
 * one-element accesses and a library-owned workspace; with both strides 1 it is
 * ks_scan.  In place (in == out and equal strides) is allowed; views
 * whose byte spans overlap otherwise are refused with KS_ERR_OVERLAP, also when
 * their elements interleave without touching.  Other arguments and errors as
 * for ks_scan.
 */
int ks_scan_strided(ks_dtype dtype, ks_op op, int inclusive, const void *in, size_t in_stride,
                    void *out, size_t out_stride, size_t n, void *stream);

/*
 * mapreduce(f, op, src) in one launch (paper Sec. II-C: op(f(src[1]), ..., f(src[n]));
 * Sec. V-A for the single-launch scheme): out[0] = f(in[0]) op f(in[1]) op ... op
 * f(in[n-1]), the left fold with the accumulated value on the left, so operators
 * that do not commute give the ordered result too (the paper requires a
 * commutative operator).  n == 0 writes the operator's identity.
 *   in    device pointer, n contiguous elements of dtype (may be NULL if n == 0)
 *   out   device pointer to ONE element of the result type, aligned to it, written
 *         by the call; it may lie inside `in`.  The result type is dtype, except
 *         where the map changes it: float for KS_MAP_UNIT_FLOAT8 and
 *         KS_MAP_WIDEN_F32, uint64_t for KS_MAP_WIDEN64 (ks_mapreduce_result_bytes
 *         gives its size)
 *   map   KS_MAP_IDENTITY or one of the maps; accepted (dtype, map, op) triples are
 *         those for which ks_mapreduce_result_bytes is not 0: every pair of
 *         ks_pair_supported, the triples of ks_map_supported, and the three sums
 *         over bytes (paper Sec. VII-B, Tables I and III):
 *         (KS_U8, KS_MAP_UNIT_FLOAT8, KS_SUM), (KS_U8, KS_MAP_WIDEN64, KS_SUM) and
 *         (KS_U8, KS_MAP_IDENTITY, KS_SUM), the last one modulo 2^8 as the element
 *         type's own addition is; and sum, minimum and maximum of 16-bit floats
 *         promoted to float, (KS_BF16 or KS_F16, KS_MAP_WIDEN_F32, KS_SUM / KS_MIN /
 *         KS_MAX), result a float.  Others return KS_ERR_UNSUPPORTED.
 * Float32 sums are accumulated in double and rounded once at the end.  Scratch,
 * stream behaviour (asynchronous; recordable into a graph under ks_scan's
 * conditions) and errors as for ks_scan; a finishing wave that does not see all
 * partial results within "spin_limit" polls leaves `out` unwritten and
 * ks_scan_check reports KS_ERR_TIMEOUT.
 */
int ks_mapreduce(ks_dtype dtype, ks_map map, ks_op op, const void *in, size_t n, void *out,
                 void *stream);

/*
 * Types and operators of the caller's own (paper Sec. IV-A, V-B: any struct of plain
 * fields, any associative operator).  The kernels are C++ templates in the headers
 * next to the library's sources (csrc/ks_launch.hpp); a translation unit of the
 * caller's, compiled by hipcc for gfx950 and linked against the library, defines
 *     struct MyOp {                         // T: a trivially copyable struct, sizeof(T) a multiple of 4
 *         static constexpr bool commutative = ...;
 *         using acc = T;                    // the type held in registers
 *         __device__ static T identity();
 *         __device__ T operator()(T earlier, T later) const;
 *     };
 *     extern "C" const void *my_pair() { return ks::Pair<T, MyOp>::entry(); }
 * and passes that pointer here.  Element sizes: 4, 8 and 16 bytes, and any other size
 * that divides 128 or 144 bytes (12, 24, 32, 36, 48, ...).  Scratch, streams, graphs,
 * errors and the in == out rule as for ks_scan and ks_mapreduce; a pointer that did
 * not come from these headers in this version returns KS_ERR_INVALID_ARG.
 * paper_2603_18695_amd/examples/user_pair.hip is a complete example.
 */
int ks_scan_pair(const void *pair, int inclusive, const void *in, void *out, size_t n, void *stream);
int ks_mapreduce_pair(const void *pair, const void *in, size_t n, void *out, void *stream);
/* sizeof the pair's element type; 0 if `pair` is not a pair of this version of the library. */
size_t ks_pair_elem_bytes(const void *pair);

/*
 * Give back the library-owned scratch that ks_scan, ks_scan_map, ks_scan_strided and
 * ks_mapreduce cache for `stream` on the current device (the pre-allocation of the
 * paper's Sec. VII-C, held until the process ends otherwise): for callers that are
 * done with a stream, or create and destroy many.  Waits for the stream first.  A
 * buffer that a stream capture has recorded is kept, since the graph may still be
 * replayed.  The next call on the stream allocates again.  Returns KS_OK also when
 * there was nothing to free.
 */
int ks_release_scratch(void *stream);

/* 1 if ks_scan_map accepts this (dtype, map, op), else 0. */
int ks_map_supported(ks_dtype dtype, ks_map map, ks_op op);

/* sizeof what ks_mapreduce writes for this (dtype, map, op); 0 if it does not accept the triple. */
size_t ks_mapreduce_result_bytes(ks_dtype dtype, ks_map map, ks_op op);

/*
 * Bytes of device scratch ks_scan_with_temp needs for this problem (the paper's
 * pre-allocation interface, Sec. VII-C).  Returns 0 for an unsupported pair or
 * bad enum.  The figure is a multiple of 256 and never 0 for a supported pair.
 */
size_t ks_scan_temp_bytes(ks_dtype dtype, ks_op op, ks_algo algo, size_t n);

/*
 * Same as ks_scan but with caller-owned scratch: `temp` is a device pointer,
 * 256-byte aligned, of at least ks_scan_temp_bytes(...) bytes, whose previous
 * contents do not matter.  Allocates nothing.  The scratch may be reused by a
 * later call on the same stream; two calls in flight at once need two buffers.
 * The call only launches kernels (the scratch is cleared by one, not by a
 * memset) and never synchronises, so it may be recorded into a HIP graph and
 * replayed.
 */
int ks_scan_with_temp(ks_dtype dtype, ks_op op, int inclusive, ks_algo algo, const void *in,
                      void *out, size_t n, void *temp, size_t temp_bytes, void *stream);

/*
 * For callers that cannot allocate device memory or own a scratch buffer: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments and errors as ks_scan, but the scratch is a static
 * device array of KS_STATIC_SCRATCH_BYTES that every device loading the library
 * holds until the process ends.  The call allocates nothing, on the device or
 * through any library, only launches kernels (the first one clears the part of
 * the array the call uses) and may be recorded into a graph.  Limit: inputs with
 * ks_scan_temp_bytes(dtype, op, KS_ALGO_AUTO, n) > KS_STATIC_SCRATCH_BYTES return
 * KS_ERR_WORKSPACE and launch nothing (8 MiB covers n up to 2^29 for float32 and 2^30
 * for the other 4-byte pairs, 2^28 for 8-byte scalars, 2^27 for the affine type and
 * 2^26 for the 16-byte types).  All calls on one device
 * share the one array: two calls that overlap in time on a device (different
 * streams, or two graphs in flight) race and give wrong results; calls on one
 * stream, one after the other, are fine.
 */
#define KS_STATIC_SCRATCH_BYTES (8u << 20)
int ks_scan_static(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n,
                   void *stream);

/*
 * Synchronise `stream` and report whether any scan issued on this stream (of
 * the current device) since the last check gave up waiting for a predecessor
 * tile (KS_ERR_TIMEOUT; that call's output is invalid), or a HIP error surfaced
 * (KS_ERR_HIP).  The stream's flag is cleared; scans on other streams have flags
 * of their own and are neither blamed nor disturbed (a device has 1024 flags,
 * handed out in order of a stream's first scan; beyond that streams share).  Waits are bounded
 * ("spin_limit") so that a scan can never hang the device: a workgroup waits
 * for tiles of workgroups that may not have started yet when other work holds
 * the compute units, and gives up if that lasts longer than the limit allows
 * (about half a second at the default).  With the option "tickets" = 1 no
 * workgroup ever waits for one that has not started.
 */
int ks_scan_check(void *stream);

/* 1 if the (dtype, op) pair is instantiated, else 0. */
int ks_pair_supported(ks_dtype dtype, ks_op op);

/* sizeof the element type, 0 for a bad enum. */
size_t ks_elem_bytes(ks_dtype dtype);

/*
 * Tuning / test knobs.  Process-wide; setting one is serialised with the calls
 * that launch, so a change never lands in the middle of a launch.
 *   "spin_limit"   polls a look-back wave makes before giving up (default 1<<20)
 *   "wgs_per_cu"   workgroups per compute unit of the persistent look-back grid:
 *                  0 = what the runtime's occupancy query reports, else 1 .. 64.
 *                  More than can be resident is safe (such grids take their tiles
 *                  by ticket), only slower
 *   "tickets"      how tiles get to workgroups: -1 = by index (workgroup b takes
 *                  tiles b, b + grid, ...) for grids of up to one workgroup per
 *                  compute unit, which is every default shape, and by ticket (a
 *                  counter in the scratch) for larger grids; 1 = always by ticket:
 *                  0-3 % slower on long inputs, more on short ones, but correct
 *                  without a timeout however long other kernels hold the device
 *   "waves"        wave64s per workgroup of the look-back kernel: 0 = the default for
 *                  the type and the input size (16 waves, one of which only looks
 *                  back, x 9 rows; for 4- and 8-byte elements 4 x 8 up to 8 MiB and
 *                  8 x 8 up to 16 MiB of input), else 4, 8 or 16
 *   "rows"         16-byte vectors per thread in the look-back kernel: 0 = the type's
 *                  default, else 4, 8, 9, 12 or 16.  A (waves, rows, prefetch, form)
 *                  combination that is not compiled for a pair makes the scan call
 *                  return KS_ERR_UNSUPPORTED: one that would not fit the register
 *                  file or LDS for the element type; and, for every pair but the
 *                  eight that the shape search runs on (sums of float, int32_t,
 *                  uint64_t and double, uint64_t maximum, the affine type, the
 *                  arg-max struct, 2x2 uint32_t matrices: all shapes that fit), one
 *                  outside what the defaults can select (16 waves in form 1 at any
 *                  rows, the pair's own default shape, 4 x 8, 8 x 8 without
 *                  prefetch, 4 x 4 for 16-byte elements)
 *   "prefetch"     1 = load the next tile before waiting in the look-back, 0 = not,
 *                  -1 = the type's default
 *   "form"         0 = one common loop for all waves (the 4- and 8-wave shapes), 1 = the
 *                  look-back wave and the data waves run loops of their own, 2 = as 1,
 *                  and every lane scans consecutive elements after an exchange through
 *                  LDS, rows 8 or 9 (1 and 2: the 16-wave shape); -1 = the default for
 *                  the pair and the input size.  A form that does not go with the
 *                  wave count gives KS_ERR_UNSUPPORTED
 * Read-only, per calling thread, what its most recent look-back launch ran:
 *   "last_grid", "last_wgs_per_cu" (the occupancy figure behind the grid),
 *   "last_waves", "last_rows", "last_form", "last_tickets"
 * ks_set_option returns KS_OK or KS_ERR_INVALID_ARG; ks_get_option the value, or -1
 * for an unknown name.
 */
int ks_set_option(const char *name, long long value);
long long ks_get_option(const char *name);

/*
 * Measurement aid (paper Sec. IV-C, the vectorised copy kernel as the practical
 * bandwidth ceiling): copy `bytes` bytes (multiple of 16, both pointers 16-byte
 * aligned) with 16-byte non-temporal loads and stores.
 */
int ks_copy(const void *in, void *out, size_t bytes, void *stream);

const char *ks_status_string(int status);
int ks_last_hip_error(void);
const char *ks_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KS_SCAN_H */
