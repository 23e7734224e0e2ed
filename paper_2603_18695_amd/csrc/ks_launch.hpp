// Host launch logic for one (element type, operator) pair: choice of kernel
// variant, grid sizing for the persistent look-back kernel, scratch layout and
// the reduce-then-scan recursion.  Instantiated once per pair in ks_pairs_*.hip.
#pragma once

#include <map>
#include <type_traits>

#include "ks_host.hpp"
#include "ks_kernels.hpp"
#include "ks_reduce.hpp"

namespace ks {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t ceil_div(size_t x, size_t y) { return (x + y - 1) / y; }

// Shape of the look-back kernel's workgroup and tile.  Measured on MI355X
// (float32 sum, n = 2^28): 4 waves x 4 rows 3.8 TB/s, 4 x 8 4.6, 4 x 16 5.2,
// 16 x 8 5.7, 16 x 9 with a dedicated look-back wave 6.2 -- the fewer and larger
// the tiles, the less the look-back costs, and one 1024-thread workgroup per
// compute unit with the next tile prefetched keeps 270 KiB of data resident per
// compute unit.
struct Shape {
    int waves, rows;
    bool prefetch;
    int form;     // kFormCommon (4 and 8 waves), kFormSeparate or kFormBlocked (16 waves)
};

// Which variants are offered at all.  A wave may use 512 / (waves per SIMD)
// registers; the tile needs 4 * ROWS * (acc size / element size) of them, the
// parked next tile 4 * ROWS, the rest goes to addresses and wave-scan temporaries.
// The bound is loose: variants close to it may spill a few registers (they stay
// correct); no default shape of any pair does (the compiler's resource report of
// every default kernel shows no scratch).
template <class T, class A, int WAVES, int ROWS, bool PREFETCH, int FORM>
constexpr bool variant_fits() {
    if (dedicated_lookback_wave(WAVES) != (FORM != kFormCommon)) return false;   // see scan_lookback_kernel
    // element sizes other than 4, 8 and 16 bytes: the blocked arrangement only, and the lane's ROWS
    // granules have to hold whole elements
    if (!granule_sized<T>() && (FORM != kFormBlocked || !blocked_fits<T, ROWS>())) return false;
    if (FORM == kFormBlocked && !blocked_fits<T, ROWS>()) return false;
    if (WAVES == 16 && ROWS == 4) return false;                   // never competitive, not compiled
    if (FORM == kFormBlocked)   // bounded by LDS; every element type compiles without spills at 8 and 9 rows
        return (size_t)(WAVES - 1) * Stage<ROWS>::SLOTS * 16 <= 150 * 1024;
    constexpr int per_wave = 512 / (WAVES / 4 > 0 ? WAVES / 4 : 1);
    constexpr int budget = per_wave > 256 ? 256 : per_wave;
    constexpr int data = 4 * ROWS * (int)(sizeof(A) / sizeof(T));
    constexpr int parked = PREFETCH ? 4 * ROWS : 0;
    // in the common loop the look-back's temporaries live next to the data, in separate loops they do not
    constexpr int other = FORM != kFormCommon ? 24 + 6 * (int)(sizeof(A) / 4) : 40 + 12 * (int)(sizeof(A) / 4);
    return data + parked + other <= budget;
}

// Default shape per pair: the best measured on MI355X, always 15 data waves + 1
// look-back wave, next tile prefetched (TB/s at 2 GiB of traffic):
//   4-byte pairs       separate loops, 9 rows                  float32 sum 6.42, int32 sum 6.38
//   8-byte sums        separate loops, 8 rows                  uint64 / float64 sum 6.43
//   8-byte min / max   separate loops, blocked arrangement   uint64 max 6.41 (striped 8 rows 6.11)
//   everything else    separate loops, blocked arrangement   affine 6.18, arg-max struct 6.25
//
// Small inputs (up to kSmallInputBytes) of 4- and 8-byte elements take 4 waves x 8
// rows instead: 32 KiB tiles spread the input over more compute units, and the run
// time of a small scan is one workgroup's load -> store latency plus the look-back
// chain.  Kernel time under rocprofv3, small against large shape: int32 sum 64 KiB
// 3.3 / 4.9 us, 256 KiB 4.2 / 5.7, 1 MiB 5.0 / 6.5, 4 MiB 6.6 / 6.8, 8 MiB 7.2 / 7.2;
// uint64 sum 64 KiB 3.9 / 4.8, 1 MiB 5.5 / 6.2, 8 MiB 7.6 / 8.3; affine 1 MiB 6.1 / 7.0.
// 16-byte elements keep the large blocked shape at every size (arg-max 64 KiB
// 6.3 / 5.9 us, 4 MiB 10.1 / 7.8: the striped scan of the small shape costs more
// than the spreading gains).
template <class T, class Op>
struct PairDefaults {
    using A = typename Op::acc;
    static constexpr bool kSum = std::is_same<typename MapOf<Op>::unmapped, SumOp<T>>::value;
    static constexpr bool kSumLike = std::is_same<typename MapOf<Op>::unmapped, SumOp<A>>::value;   // a sum of the accumulator type
    static constexpr Shape shape() {
        if (!granule_sized<T>()) return Shape{16, blocked_fits<T, 9>() ? 9 : 8, true, kFormBlocked};
        // 2-byte elements accumulated in 4 bytes: a granule unpacks into eight registers, and 8 rows of
        // them with the parked next tile are what 128 registers hold
        if (sizeof(T) == 2) return Shape{16, 8, true, kFormSeparate};
        if (sizeof(A) == 4) return Shape{16, 9, true, kFormSeparate};
        // 8-byte scalars, sums: 8 rows in striped separate loops measure 1 % above 9 rows blocked
        // (uint64 sum 6.32 / 6.26, float64 sum 6.33 / 6.26 TB/s).  Minimum and maximum of 8-byte values
        // take several instructions per combination, and the striped arrangement pays them in one
        // wave scan per row: blocked 9 rows is 5 % ahead (uint64 max 6.41 / 6.11, float64 min 6.40 / 6.07).
        if (sizeof(A) == 8 && sizeof(T) == 8 && kSum) return Shape{16, 8, true, kFormSeparate};
        return Shape{16, 9, true, kFormBlocked};
    }
    static constexpr Shape small_shape() { return Shape{4, 8, true, kFormCommon}; }
    static constexpr size_t kSmallInputBytes = (size_t)8 << 20;
    // Between the two, 8 waves x 8 rows (64 KiB tiles, no next tile to prefetch): up to 34 MiB the
    // large tile leaves compute units without work (16 MiB are 124 tiles of 135 KiB).  Against the
    // large shape, TB/s: int32 sum 16 MiB 3.48 / 3.18, uint64 sum 16 MiB 3.35 / 3.07, 32 MiB 5.11 / 4.75;
    // from 32 MiB (4-byte) and 64 MiB (8-byte elements) on the large shape is ahead.  That was the
    // large shape before its pauses; with them 8-byte scalars are ahead in 16 waves x 8 rows from 16 MiB
    // on (uint64 sum, us per call, 8 x 8 / 16 x 8: 20 MiB 10.8 / 10.0, 24 MiB 12.3 / 10.4, 28 MiB 12.8 / 11.6).
    // Not for pairs that accumulate wider than they store (the affine type, float32 in, float64
    // accumulators): its common loop is slow for them (8 x 8 / blocked 16 x 9, us per call: 14 MiB
    // 11.1 / 10.8, 20 MiB 18.0 / 11.5, 32 MiB 21.1 / 14.5).
    static constexpr Shape mid_shape() { return Shape{8, 8, false, kFormCommon}; }
    static constexpr size_t kMidInputBytes = sizeof(A) == sizeof(T) ? (size_t)16 << 20 : kSmallInputBytes;
    // 16-byte elements: only up to 1 MiB a small tile wins, 4 waves x 4 rows (kernel time against
    // the large blocked shape: quaternions 64 KiB 5.0 / 5.9 us, 1 MiB 6.6 / 7.9; arg-max struct
    // 1 MiB 6.8 / 7.4; at 4 MiB the blocked shape is ahead, 7.7 / 8.8).
    static constexpr size_t kSmallInputBytes16 = (size_t)1 << 20;
    static constexpr Shape shape_for(size_t n) {
        if (!granule_sized<T>()) return shape();   // one shape at every size
        if (sizeof(T) >= 16 && n * sizeof(T) <= kSmallInputBytes16) return Shape{4, 4, true, kFormCommon};
        if (sizeof(T) < 16 && n * sizeof(T) <= kSmallInputBytes) return small_shape();
        if (sizeof(T) < 16 && n * sizeof(T) <= kMidInputBytes) return mid_shape();
        return shape();
    }
};

// Which pairs are compiled in EVERY shape that fits: the subjects of the shape search, one or two per
// element class (their results set the class's defaults).  Every other pair is compiled in the
// shapes its defaults can select: the 16-wave shapes in separate loops (all rows: inputs of a few
// rounds choose among them), its own default shape, and the small shapes 4 x 8, 8 x 8 and 4 x 4.
// A shape option that asks for anything else is refused for them with KS_ERR_UNSUPPORTED.  The full
// matrix is some sixty kernels per pair, the reduced one some twenty.
template <class T, class Op>
struct FullMatrix : std::false_type {};
template <> struct FullMatrix<float, SumOp<float>> : std::true_type {};
template <> struct FullMatrix<int32_t, SumOp<int32_t>> : std::true_type {};
template <> struct FullMatrix<uint64_t, SumOp<uint64_t>> : std::true_type {};
template <> struct FullMatrix<double, SumOp<double>> : std::true_type {};
template <> struct FullMatrix<uint64_t, MaxOp<uint64_t>> : std::true_type {};
template <> struct FullMatrix<AffineF32, AffineComposeOp> : std::true_type {};
template <> struct FullMatrix<ArgmaxI32Cnt64, ArgmaxCountOp> : std::true_type {};
template <> struct FullMatrix<Mat2U32, Mat2MulOp> : std::true_type {};

template <class T, class Op, int WAVES, int ROWS, bool PREFETCH, int FORM>
constexpr bool variant_offered() {
    if (!variant_fits<T, typename Op::acc, WAVES, ROWS, PREFETCH, FORM>()) return false;
    if (FullMatrix<T, Op>::value) return true;
    constexpr Shape d = PairDefaults<T, Op>::shape();
    if (WAVES == 16) return FORM == kFormSeparate || (FORM == d.form && ROWS == d.rows);
    if (WAVES == 4) return (ROWS == 8 && PREFETCH) || (ROWS == 4 && PREFETCH && sizeof(T) >= 16);
    return WAVES == 8 && ROWS == 8 && !PREFETCH;
}

// Workgroups per compute unit the runtime reports for a kernel variant, per device.  It can be
// higher than what the hardware grants; with tickets that only means some workgroups start late.
template <class Kernel>
inline int reported_occupancy(const ScanCall &c, std::map<int, int> &cache, Kernel kernel, int threads, int &per_cu) {
    int &known = cache[c.dev->device];
    if (known == 0) {
        int nb = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, threads, 0);
        if (e != hipSuccess) return set_hip_error(e);
        known = nb > 0 ? nb : 1;
    }
    per_cu = known;
    return KS_OK;
}

// ---- mapreduce: the launch -----------------------------------------------------------
// Every pair can be reduced; those that are also scanned reach this through Pair, the byte types
// through ReducePair.
template <class T, class Op>
struct ReduceLaunch {
    using C = typename ChainOf<Op>::type;
    using R = typename ResultOf<Op, T>::type;
    // c.out points to ONE element; c.temp holds the control block and the workgroups' partials.
    // Shape, measured on MI355X (GB/s of the bytes read, rows x workgroups per compute unit).  Commutative
    // operators (strided runs): float32 sum 2^28 4 x 2 7186, 2 x 4 6970, 4 x 4 6876, 8 x 2 6871, 4 x 8 6459;
    // arg-max struct 2^26 4 x 2 7120, 4 x 4 6771, 4 x 8 6344: two workgroups per compute unit keep enough
    // loads in flight, more only add partials to fold at the end.  Ordered reductions (contiguous
    // ranges, blocked arrangement through LDS, one ordered wave reduction per run; 8 rows, 9 for the
    // 12-byte struct), us per call with 1 / 2 / 3 workgroups per compute unit:
    //   affine (8 bytes)        128 MiB 24.3 / 24.9 / 29.4   512 MiB 79.8 / 84.1 / 88.9   1 GiB 180 / 160 / 174   2 GiB 349 / 332 / 337
    //   range struct (12 bytes) 128 MiB 22.2 / 24.0 / 26.2   512 MiB 78.1 / 80.5 / 83.2   1 GiB 151 / 158 / 166   2 GiB 308 / 310 / 325
    //   2x2 uint32 matrices     128 MiB 26.1 / 25.6 / 30.1   512 MiB 85.3 / 83.3 / 91.0   1 GiB 179 / 160 / 175   2 GiB 332 / 334 / 338
    //   quaternions             128 MiB 28.7 / 26.5 / 30.8   512 MiB 93.9 / 84.8 / 92.7   1 GiB 195 / 160 / 176   2 GiB 366 / 336 / 337
    //   2x2 uint64 matrices     128 MiB 37.9 / 31.9 / 35.4   512 MiB 126 / 89.7 / 97.5    1 GiB 242 / 173 / 180   2 GiB 457 / 340 / 335
    // so: two, but one for elements below 16 bytes up to 768 MiB (for the 12-byte struct at any size).
    static constexpr bool kOrdered = ordered_reduction<T, Op>();
    static constexpr int kReduceRows = !kOrdered ? 4 : blocked_fits<T, 8>() ? 8 : 9;
    // Bytes decoded to float32 (UnitFloat8): five instructions per byte read make that kernel bound by
    // arithmetic, and a third workgroup per compute unit hides more of it: n = 10^9, us per call with
    // 1 / 2 / 3 / 4 / 6 workgroups 285 / 176 / 151 / 151 / 160 (10^8: 32 / 23.7 / 24.2 / 27 / 31); the plain
    // byte sums stay at two: 220 / 138 / 146 / 147 / 151.
    static constexpr bool kDecodesBytes = sizeof(T) == 1 && std::is_same<typename Op::acc, float>::value;
    static constexpr int kReduceWgsPerCu = kDecodesBytes ? 3 : 2;
    static constexpr bool kOneWhenSmall = kOrdered && sizeof(T) < 16;
    static constexpr size_t kReduceRun = (size_t)kWave * kReduceRows * 16 / sizeof(T);   // elements per run
    static size_t reduce_scratch_bytes(size_t grid) {
        return kControlBytes + align_up((grid > 0 ? grid : 1) * WordsOf<C>::W * sizeof(uint64_t), 256);
    }
    static int run(const ScanCall &c) {
        auto kernel = mapreduce_kernel<T, Op, kReduceRows>;
        static std::map<int, int> reported_per_cu;
        int per_cu = 0;
        const int os = reported_occupancy(c, reported_per_cu, kernel, kBlock, per_cu);
        if (os != KS_OK) return os;
        if (per_cu > kReduceWgsPerCu) per_cu = kReduceWgsPerCu;
        if (kOneWhenSmall && (c.n * sizeof(T) < ((size_t)768 << 20) || sizeof(T) % 8 != 0)) per_cu = 1;
        const long long want = options().wgs_per_cu;
        if (want > 0) per_cu = (int)(want < 64 ? want : 64);   // any grid is safe here: nobody waits for a workgroup
        // Elements narrower than a dword: the kernel's 16-byte reads start on a dword boundary, so the
        // input is taken from the boundary at or below `in` (the same dword, hence the same
        // allocation) and the kernel drops the bytes in front of the first element.
        const T *in = static_cast<const T *>(c.in);
        size_t n = c.n;
        uint32_t head_skip = 0;
        if (sizeof(T) < 4 && n > 0) {
            head_skip = (uint32_t)(reinterpret_cast<uintptr_t>(in) & 3u);
            in = reinterpret_cast<const T *>(reinterpret_cast<uintptr_t>(in) - head_skip);
            n += head_skip / sizeof(T);
        }
        const size_t total_runs = ceil_div(n, kReduceRun);
        size_t grid = (size_t)per_cu * (size_t)c.dev->cus;
        // The full grid at every size: with the arrivals counted in two levels (ks_reduce.hpp) a workgroup
        // costs next to nothing at the end.  float32 sum, us per call from C, 1 / 2 workgroups per compute
        // unit: 4 MB 4.1 / 4.1, 10 MB 5.2 / 4.8, 20 MB 6.9 / 5.9, 40 MB 10.6 / 8.5, 100 MB 21.3 / 16.6, 400 MB 75 / 58.
        // (Counted on one word, 512 workgroups cost 5 us at the end, and grids had to shrink with the input.)
        if (grid > ceil_div(total_runs, (size_t)kWaves)) grid = ceil_div(total_runs, (size_t)kWaves);
        if (grid < 1) grid = 1;   // n == 0: one workgroup writes the identity
        if (reduce_scratch_bytes(grid) > c.temp_bytes) return KS_ERR_WORKSPACE;
        char *base = static_cast<char *>(c.temp);
        if (c.clear_descriptors) {
            const size_t words = reduce_scratch_bytes(grid) / sizeof(uint64_t);
            hipLaunchKernelGGL((fill_zero_kernel<0>), dim3((unsigned)ceil_div(words, 256)), dim3(256), 0, c.stream,
                               reinterpret_cast<uint64_t *>(base), words);
        }
        ReduceArgs a;
        a.n = n;
        a.head_skip = head_skip;
        a.total_runs = total_runs;
        a.control = reinterpret_cast<uint32_t *>(base);
        a.partials = reinterpret_cast<uint64_t *>(base + kControlBytes);
        a.epoch = c.epoch;
        long long spin = options().spin_limit;
        a.spin_limit = (uint32_t)(spin < 0 ? 0 : (spin > 0xffffffffll ? 0xffffffffll : spin));
        a.abort_flag = c.abort_flag;
        a.call_seq = c.call_seq;
        // Ordered reductions: an odd number of runs per wave.  All waves walk their ranges in step, and
        // with ranges a power of two apart (1 GiB over 1024 waves: 1 MiB) their reads fall on the
        // same memory channels at the same time (affine, 1 GiB: 178 us against 163 us with ranges 512 KiB apart).
        size_t per_wave = ceil_div(total_runs, grid * kWaves);
        if (per_wave > 2) per_wave |= 1;
        if (per_wave > 0xffffffffull) return KS_ERR_INVALID_ARG;
        a.runs_per_wave = (uint32_t)per_wave;
        LastLaunch &l = last_launch();
        l.grid = (long long)grid;
        l.wgs_per_cu = per_cu;
        l.waves = kWaves;
        l.rows = kReduceRows;
        l.form = kFormCommon;
        l.tickets = 0;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kBlock), 0, c.stream, in, static_cast<R *>(c.out), a);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? KS_OK : set_hip_error(e);
    }
};

// T = element type in memory; A = Op::acc = type held in registers; C = the operator's chain type =
// type of aggregates, seeds and descriptors.
template <class T, class Op>
struct Pair {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    static constexpr int W = WordsOf<C>::W;
    // The reduce-then-scan kernels run 4 waves x 4 rows in the striped arrangement; element sizes
    // other than 4, 8 and 16 bytes take the blocked arrangement with the rows of their look-back shape.
    static constexpr bool kRtsBlocked = !granule_sized<T>();
    static constexpr int kRtsRows = kRtsBlocked ? PairDefaults<T, Op>::shape().rows : 4;
    static constexpr int kMinTileGranules = 4 * kWave * 4;   // smallest compiled look-back tile: 4 waves x 4 rows

    // elements in `granules` 16-byte granules (callers pass whole tiles, which hold whole elements)
    static size_t granule_elems(size_t granules) { return granules * 16 / sizeof(T); }
    static size_t tile_elems(int rows) { return granule_elems((size_t)kWaves * kWave * rows); }
    static size_t shape_tile_elems(int waves, int rows) { return granule_elems((size_t)data_waves(waves) * kWave * rows); }

    static size_t desc_bytes(size_t count) { return align_up((count > 0 ? count : 1) * W * sizeof(uint64_t), 256); }

    // Inputs of up to three rounds of the default tile (one tile per compute unit and round): the
    // workgroups move in lock-step there (the staggered start begins at three rounds), so the run time
    // goes with rounds x rows per thread, and a last round with a few tiles costs as much as a full
    // one.  Take the rows that minimise that product; the default stays on a tie.  Measured, us per
    // call, default rows / chosen rows: float32 sum 40 MiB 17.8 / 15.5 (12 rows, one round), 48 MiB
    // 20.1 / 18.3 (16 rows, one round), 72 MiB 29.2 / 26.3 (12 rows, two rounds instead of three), 80 MiB
    // 32.0 / 28.9; uint64 sum 40 MiB 18.0 / 16.1 (12 rows), 64 MiB 26.9 / 23.2 (9 rows, two rounds instead
    // of three); 16 rows in one round against 8 rows in two is a tie by the product and measures
    // worse (uint64 48 MiB 22.3 against 18.6), hence the tie rule.  The same product sends 4-byte
    // inputs of less than one round of 8-row tiles to 8 rows (float32 sum 24 MiB 11.3 / 10.6, 28 MiB
    // 12.2 / 11.4).  Elements of 16 bytes keep their blocked shape.
    static Shape few_rounds_shape(size_t n, int cus, Shape s) {
        if (sizeof(T) >= 16 || s.waves != 16 || s.rows > 9) return s;
        auto rounds = [&](int rows) { return ceil_div(ceil_div(n, shape_tile_elems(16, rows)), (size_t)cus); };
        const size_t r0 = rounds(s.rows);
        if (r0 > 3) return s;
        Shape best = s;
        size_t best_cost = r0 * (size_t)s.rows;
        auto consider = [&](Shape c) {
            const size_t cost = rounds(c.rows) * (size_t)c.rows;
            if (cost < best_cost) {
                best = c;
                best_cost = cost;
            }
        };
        if (s.rows == 8 && s.form == kFormSeparate && variant_fits<T, A, 16, 9, true, kFormSeparate>())
            consider(Shape{16, 9, true, kFormSeparate});
        if (variant_fits<T, A, 16, 12, true, kFormSeparate>())
            consider(Shape{16, 12, true, kFormSeparate});
        else if (variant_fits<T, A, 16, 12, false, kFormSeparate>() && (sizeof(T) > 2 || PairDefaults<T, Op>::kSumLike))
            consider(Shape{16, 12, false, kFormSeparate});   // (16-bit minimum / maximum: five registers over at 12 rows)
        if (variant_fits<T, A, 16, 16, false, kFormSeparate>() && rounds(16) == 1)
            consider(Shape{16, 16, false, kFormSeparate});
        // less than one round: smaller tiles keep more compute units busy
        if (s.rows == 9 && sizeof(A) == 4 && variant_fits<T, A, 16, 8, true, kFormSeparate>())
            consider(Shape{16, 8, true, kFormSeparate});
        // one round: there is no next tile to park, and the kernel without the parking registers is
        // the leaner one (float32 sum n = 10^7 in 12 rows: 15.5 us against 21.7 us)
        if (rounds(best.rows) == 1) best.prefetch = false;
        return best;
    }

    static Shape lookback_shape(size_t n, int cus) {
        Shape s = PairDefaults<T, Op>::shape_for(n);
        s = few_rounds_shape(n, cus, s);
        const Options &o = options();
        if (o.waves == 4 || o.waves == 8 || o.waves == 16) s.waves = (int)o.waves;
        if (o.rows == 4 || o.rows == 8 || o.rows == 9 || o.rows == 12 || o.rows == 16) s.rows = (int)o.rows;
        if (o.prefetch >= 0) s.prefetch = o.prefetch != 0;
        // an explicit wave count takes the form that goes with it; an explicit form that does not go
        // with the wave count is refused by the dispatch below
        if (!dedicated_lookback_wave(s.waves)) s.form = kFormCommon;
        else if (s.form == kFormCommon) s.form = PairDefaults<T, Op>::shape().form;
        if (o.form >= 0) s.form = (int)o.form;
        return s;
    }

    static ks_algo pick_algo(size_t n) {
        // one tile: a single workgroup scans it directly (handled inside the reduce-then-scan path)
        if (n <= tile_elems(kRtsRows)) return KS_ALGO_REDUCE_THEN_SCAN;
        return KS_ALGO_LOOKBACK;
    }

    static size_t temp_bytes(ks_algo algo, size_t n) {
        if (algo == KS_ALGO_AUTO) algo = pick_algo(n);
        if (algo == KS_ALGO_LOOKBACK) {
            // sized for the smallest tile any compiled variant uses, so a later change of the
            // shape options cannot outgrow a buffer sized earlier
            const size_t tiles = ceil_div(n * sizeof(T), (size_t)kMinTileGranules * 16);
            return lookback_scratch_bytes(tiles + 1);   // + 1: tile 0 may be cut short (output-aligned tiles)
        }
        size_t total = 0, m = n;
        const size_t tile = tile_elems(kRtsRows);
        if (m > tile) {
            m = ceil_div(m, tile);
            total = align_up(m * sizeof(C), 256);
            using Upper = Pair<C, typename ChainOf<Op>::op>;
            if (m > Upper::tile_elems(Upper::kRtsRows)) total += Upper::temp_bytes(KS_ALGO_REDUCE_THEN_SCAN, m);
        }
        return total > 0 ? total : 256;
    }

    // ---- look-back ---------------------------------------------------------
    // Scratch of a look-back call: control block, D descriptors, X descriptors.
    static size_t lookback_scratch_bytes(size_t tiles) {
        return kControlBytes + desc_bytes(tiles) + desc_bytes(ceil_div(tiles, kWindow) * kWindow);
    }

    // grid of a persistent look-back launch, and whether first tiles come from tickets as well
    static size_t persistent_grid(const ScanCall &c, int per_cu, size_t tiles, uint32_t &tickets) {
        const long long want = options().wgs_per_cu;
        const int use = want > 0 ? (int)(want < 64 ? want : 64) : per_cu;
        size_t grid = (size_t)use * (size_t)c.dev->cus;
        if (grid > tiles) grid = tiles;
        // up to one workgroup per compute unit every workgroup is sure to run, whatever else the
        // device is doing: tiles by index (see "Tile assignment" in ks_kernels.hpp)
        tickets = grid > (size_t)c.dev->cus || options().tickets == 1 ? 1u : 0u;
        LastLaunch &l = last_launch();
        l.grid = (long long)grid;
        l.wgs_per_cu = per_cu;
        l.tickets = tickets;
        return grid;
    }
    // Fills in everything of the kernel's arguments that the data pointers do not cover; clears the
    // scratch first if its contents are unknown.
    static LookbackArgs lookback_args(const ScanCall &c, size_t tiles, uint32_t tickets) {
        char *base = static_cast<char *>(c.temp);
        if (c.clear_descriptors) {
            const size_t words = lookback_scratch_bytes(tiles) / sizeof(uint64_t);
            const unsigned fb = (unsigned)(ceil_div(words, 256) < 1024 ? ceil_div(words, 256) : 1024);
            hipLaunchKernelGGL((fill_zero_kernel<0>), dim3(fb), dim3(256), 0, c.stream, reinterpret_cast<uint64_t *>(base), words);
        }
        LookbackArgs a;
        a.n = c.n;
        a.control = reinterpret_cast<uint32_t *>(base);
        a.desc = reinterpret_cast<uint64_t *>(base + kControlBytes);
        a.xdesc = a.desc + desc_bytes(tiles) / sizeof(uint64_t);
        a.epoch = c.epoch;
        a.ntiles = (uint32_t)tiles;
        long long spin = options().spin_limit;
        if (spin < 0) spin = 0;
        if (spin > 0xffffffffll) spin = 0xffffffffll;
        a.spin_limit = (uint32_t)spin;
        a.abort_flag = c.abort_flag;
        a.call_seq = c.call_seq;
        a.tickets = tickets;
        a.seeded = 0;
        return a;
    }

    template <int WAVES, int ROWS, bool INCLUSIVE, bool PREFETCH, int FORM>
    static int launch_lookback(const ScanCall &c) {
        if constexpr (!variant_offered<T, Op, WAVES, ROWS, PREFETCH, FORM>()) {
            return KS_ERR_UNSUPPORTED;   // would spill registers for this element type, or is not compiled for this pair
        } else {
            auto kernel = scan_lookback_kernel<T, Op, WAVES, ROWS, INCLUSIVE, PREFETCH, FORM>;
            constexpr int kThreads = WAVES * kWave;
            // kernels that move their tiles to the output's line boundaries have tile 0 cut short
            const size_t shift = aligns_output(WAVES)
                                     ? tile_shift(static_cast<const T *>(c.out), shape_tile_elems(WAVES, ROWS))
                                     : 0;
            const size_t tiles = ceil_div(c.n + shift, shape_tile_elems(WAVES, ROWS));
            if (tiles >= 0xfffffff0ull) return KS_ERR_INVALID_ARG;   // tile indices and tickets are 32-bit
            if (lookback_scratch_bytes(tiles) > c.temp_bytes) return KS_ERR_WORKSPACE;
            static std::map<int, int> reported_per_cu;
            int per_cu = 0;
            const int os = reported_occupancy(c, reported_per_cu, kernel, kThreads, per_cu);
            if (os != KS_OK) return os;
            uint32_t tickets = 0;
            const size_t grid = persistent_grid(c, per_cu, tiles, tickets);
            LastLaunch &l = last_launch();
            l.waves = WAVES;
            l.rows = ROWS;
            l.form = FORM;
            LookbackArgs a = lookback_args(c, tiles, tickets);
            if (c.seed) {   // after the scratch has been cleared (if it had to be), before the scan starts
                hipLaunchKernelGGL((seed_store_kernel<T, Op>), dim3(1), dim3(kWave), 0, c.stream,
                                   static_cast<const T *>(c.seed), a.control);
                a.seeded = 1;
            }
            hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kThreads), 0, c.stream,
                               static_cast<const T *>(c.in), static_cast<T *>(c.out), a);
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? KS_OK : set_hip_error(e);
        }
    }

    template <int WAVES, int ROWS, int FORM>
    static int lookback_flags_dispatch(const ScanCall &c, bool pf) {
        if (c.inclusive)
            return pf ? launch_lookback<WAVES, ROWS, true, true, FORM>(c) : launch_lookback<WAVES, ROWS, true, false, FORM>(c);
        return pf ? launch_lookback<WAVES, ROWS, false, true, FORM>(c) : launch_lookback<WAVES, ROWS, false, false, FORM>(c);
    }

    template <int WAVES, int ROWS>
    static int lookback_pf_dispatch(const ScanCall &c, const Shape &s) {
        if constexpr (dedicated_lookback_wave(WAVES)) {
            if (s.form == kFormBlocked) return lookback_flags_dispatch<WAVES, ROWS, kFormBlocked>(c, s.prefetch);
            if (s.form == kFormSeparate) return lookback_flags_dispatch<WAVES, ROWS, kFormSeparate>(c, s.prefetch);
        } else {
            if (s.form == kFormCommon) return lookback_flags_dispatch<WAVES, ROWS, kFormCommon>(c, s.prefetch);
        }
        return KS_ERR_UNSUPPORTED;   // the 16-wave shape has no common loop, the others nothing to separate
    }

    template <int WAVES>
    static int lookback_rows_dispatch(const ScanCall &c, const Shape &s) {
        switch (s.rows) {
            case 4: return lookback_pf_dispatch<WAVES, 4>(c, s);
            case 8: return lookback_pf_dispatch<WAVES, 8>(c, s);
            case 9: return lookback_pf_dispatch<WAVES, 9>(c, s);
            case 12: return lookback_pf_dispatch<WAVES, 12>(c, s);
            case 16: return lookback_pf_dispatch<WAVES, 16>(c, s);
            default: return KS_ERR_INVALID_ARG;
        }
    }

    static int run_lookback(const ScanCall &c) {
        const Shape s = lookback_shape(c.n, c.dev->cus);
        switch (s.waves) {
            case 4: return lookback_rows_dispatch<4>(c, s);
            case 8: return lookback_rows_dispatch<8>(c, s);
            case 16: return lookback_rows_dispatch<16>(c, s);
            default: return KS_ERR_INVALID_ARG;
        }
    }

    // ---- reduce-then-scan ----------------------------------------------------
    static int launch_tile_scan(bool inclusive, const T *in, T *out, size_t n, const C *seeds, hipStream_t s) {
        const size_t tiles = ceil_div(n, tile_elems(kRtsRows));
        if (inclusive)
            hipLaunchKernelGGL((tile_scan_kernel<T, Op, kRtsRows, true, kRtsBlocked>), dim3((unsigned)tiles), dim3(kBlock), 0, s, in,
                               out, n, seeds);
        else
            hipLaunchKernelGGL((tile_scan_kernel<T, Op, kRtsRows, false, kRtsBlocked>), dim3((unsigned)tiles), dim3(kBlock), 0, s,
                               in, out, n, seeds);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? KS_OK : set_hip_error(e);
    }

    static int run_rts(bool inclusive, const T *in, T *out, size_t n, char *temp, size_t temp_bytes, hipStream_t s) {
        const size_t tile = tile_elems(kRtsRows);
        const size_t tiles = ceil_div(n, tile);
        if (tiles <= 1) return launch_tile_scan(inclusive, in, out, n, nullptr, s);
        const size_t need = align_up(tiles * sizeof(C), 256);
        if (need > temp_bytes) return KS_ERR_WORKSPACE;
        C *agg = reinterpret_cast<C *>(temp);
        hipLaunchKernelGGL((tile_reduce_kernel<T, Op, kRtsRows, kRtsBlocked>), dim3((unsigned)tiles), dim3(kBlock), 0, s, in, n, agg);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return set_hip_error(e);
        // aggregates -> exclusive prefixes of the tiles, in place (scratch is 256-byte aligned)
        // (the map has been applied by the reduction; the levels above combine plain accumulators)
        using Upper = Pair<C, typename ChainOf<Op>::op>;
        int st = Upper::run_rts(false, agg, agg, tiles, temp + need, temp_bytes - need, s);
        if (st != KS_OK) return st;
        return launch_tile_scan(inclusive, in, out, n, agg, s);
    }

    // ---- strided views -------------------------------------------------------
    // The look-back scan with element-wise accesses and one-element granules, WAVES waves x
    // strided_rows rows x 64 elements per tile; one tile or many.  One workgroup per compute unit,
    // tiles by index.
    // Rows: 16, 8 or 4 by the accumulator's size.  The 16-wave workgroup has 128 registers per lane,
    // and the items and their lane bases (2 x rows x the accumulator's words) stay live across the
    // look-back: half the rows for accumulators of 8 bytes and more, 12 for the float32 sum, whose
    // look-back runs in double.
    template <int WAVES>
    static constexpr int strided_rows() {
        constexpr int base = sizeof(A) >= 32 ? 4 : sizeof(A) >= 16 ? 8 : 16;
        if (WAVES < 16) return base;
        if (sizeof(A) >= 8) return base / 2;
        return sizeof(C) > sizeof(A) ? 12 : base;
    }
    template <int WAVES>
    static constexpr size_t strided_tile() { return (size_t)WAVES * kWave * strided_rows<WAVES>(); }
    // temp_bytes(KS_ALGO_LOOKBACK, n) sizes the descriptors for the smallest contiguous tile
    static_assert(sizeof(T) < 4 ||   // 2-byte elements are not scanned through strided views (run_strided)
                      (strided_tile<4>() * sizeof(T) >= (size_t)kMinTileGranules * 16 &&
                       strided_tile<8>() * sizeof(T) >= (size_t)kMinTileGranules * 16 &&
                       strided_tile<16>() * sizeof(T) >= (size_t)kMinTileGranules * 16),
                  "strided tile below the smallest tile");
    template <int WAVES, bool INCLUSIVE>
    static int launch_lookback_strided(const ScanCall &c) {
        auto kernel = scan_lookback_strided_kernel<T, Op, WAVES, strided_rows<WAVES>(), INCLUSIVE>;
        constexpr int kThreads = WAVES * kWave;
        const size_t tiles = ceil_div(c.n, strided_tile<WAVES>());
        if (tiles >= 0xfffffff0ull) return KS_ERR_INVALID_ARG;
        if (lookback_scratch_bytes(tiles) > c.temp_bytes) return KS_ERR_WORKSPACE;
        uint32_t tickets = 0;
        const size_t grid = persistent_grid(c, 1, tiles, tickets);
        LastLaunch &l = last_launch();
        l.waves = WAVES;
        l.rows = strided_rows<WAVES>();
        l.form = kFormCommon;
        const LookbackArgs a = lookback_args(c, tiles, tickets);
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kThreads), 0, c.stream, static_cast<const T *>(c.in),
                           c.in_stride, static_cast<T *>(c.out), c.out_stride, a);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? KS_OK : set_hip_error(e);
    }
    // Workgroup size by the distance between neighbouring elements: the closer they are, the more
    // of each cache line a wave uses and the more waves a compute unit can feed.  Measured, n = 2^24,
    // us per call with 4 / 8 / 16 waves: float32 stride 2 (8 bytes apart) 99 / 73 / 64, stride 4 160 / 151 /
    // 163, stride 8 287 / 290 / 332, stride 32 1109 / 1121 / 1169; float64 stride 2 (16 bytes) 161 / 152 / 204,
    // stride 4 294 / 295 / 404, stride 8 593 / 637 / 763.
    static int run_strided(const ScanCall &c) {
        if constexpr (sizeof(T) < 4) return KS_ERR_UNSUPPORTED;   // one-element accesses below a dword: not built
        else return run_strided_views(c);
    }
    static int run_strided_views(const ScanCall &c) {
        const size_t apart = (c.in_stride > c.out_stride ? c.in_stride : c.out_stride) * sizeof(T);
        int waves = apart <= 8 ? 16 : apart <= 16 ? 8 : 4;
        const long long want = options().waves;
        if (want == 4 || want == 8 || want == 16) waves = (int)want;
        switch (waves) {
            case 4: return c.inclusive ? launch_lookback_strided<4, true>(c) : launch_lookback_strided<4, false>(c);
            case 8: return c.inclusive ? launch_lookback_strided<8, true>(c) : launch_lookback_strided<8, false>(c);
            default:
                // elements of 8 bytes and more are never 8 bytes apart, so only the "waves" option leads
                // here for them; with more than 8 bytes to accumulate the wave scans do not fit 128 registers: not compiled
                if constexpr (sizeof(T) > 8 || sizeof(A) > 8) return KS_ERR_UNSUPPORTED;
                else return c.inclusive ? launch_lookback_strided<16, true>(c) : launch_lookback_strided<16, false>(c);
        }
    }

    // ---- mapreduce ---------------------------------------------------------------
    static int run_mapreduce(const ScanCall &c) { return ReduceLaunch<T, Op>::run(c); }

    static int run(const ScanCall &c) {
        if (c.in_stride != 1 || c.out_stride != 1)
            return run_strided(c);
        if (c.algo == KS_ALGO_LOOKBACK) return run_lookback(c);
        return run_rts(c.inclusive != 0, static_cast<const T *>(c.in), static_cast<T *>(c.out), c.n,
                       static_cast<char *>(c.temp), c.temp_bytes, c.stream);
    }

    static const PairEntry *entry() {
        // scans of 2-byte elements work on whole dwords: both arrays start on one
        constexpr size_t align = sizeof(T) < 4 ? 4 : alignof(T);
        static const PairEntry e = {kPairAbi, sizeof(T), align, &Pair::temp_bytes, &Pair::pick_algo, &Pair::run,
                                    &Pair::run_mapreduce, sizeof(T), align};
        return &e;
    }
};

// A pair that is only reduced: its elements are narrower than the scan kernels' 4 bytes.
template <class T, class Op>
struct ReducePair {
    static const PairEntry *entry() {
        static const PairEntry e = {kPairAbi, sizeof(T), alignof(T), nullptr, nullptr, nullptr, &ReduceLaunch<T, Op>::run,
                                    sizeof(typename ResultOf<Op, T>::type), alignof(typename ResultOf<Op, T>::type)};
        return &e;
    }
};

}  // namespace ks
