// Host launch logic for one (element type, operator) pair: choice of kernel
// variant, grid sizing for the persistent look-back kernel, scratch layout and
// the reduce-then-scan recursion.  Instantiated once per pair in ks_pairs_*.hip.
#pragma once

#include "ks_host.hpp"
#include "ks_kernels.hpp"

namespace ks {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t ceil_div(size_t x, size_t y) { return (x + y - 1) / y; }

// Measured on MI355X for every element size: the largest compiled tile with the
// next tile prefetched wins (fewer tiles, fewer look-backs, longer streams
// between synchronisations), even though it leaves only 2 workgroups per
// compute unit resident.  Types whose accumulator is wider than the element in
// memory run out of registers earlier and stop at 8 rows.
template <class T, class A>
struct PairDefaults {
    static constexpr int rows = sizeof(A) > sizeof(T) ? 8 : 16;
    static constexpr bool prefetch = true;
};

// T = element type in memory; A = Op::acc = type of aggregates, seeds and descriptors.
template <class T, class Op>
struct Pair {
    using A = typename Op::acc;
    static constexpr int W = WordsOf<A>::W;
    static constexpr int kRtsRows = 4;

    static size_t tile_elems(int rows) { return (size_t)kWaves * kWave * rows * (16 / sizeof(T)); }

    static size_t desc_bytes(size_t count) { return align_up((count > 0 ? count : 1) * W * sizeof(uint64_t), 256); }

    static int lookback_rows() {
        const long long r = options().rows;
        return (r == 2 || r == 4 || r == 8 || r == 16) ? (int)r : PairDefaults<T, A>::rows;
    }
    static bool lookback_prefetch() {
        const long long p = options().prefetch;
        return p < 0 ? PairDefaults<T, A>::prefetch : p != 0;
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
            // "rows" option cannot outgrow a buffer sized earlier
            const size_t tiles = ceil_div(n, tile_elems(2));
            return desc_bytes(tiles) + desc_bytes(ceil_div(tiles, kWindow) * kWindow);
        }
        size_t total = 0, m = n;
        const size_t tile = tile_elems(kRtsRows);
        if (m > tile) {
            m = ceil_div(m, tile);
            total = align_up(m * sizeof(A), 256);
            if (m > Pair<A, Op>::tile_elems(kRtsRows)) total += Pair<A, Op>::temp_bytes(KS_ALGO_REDUCE_THEN_SCAN, m);
        }
        return total > 0 ? total : 256;
    }

    // ---- look-back ---------------------------------------------------------
    template <int ROWS, bool INCLUSIVE, bool PREFETCH>
    static int launch_lookback(const ScanCall &c, int aligned) {
        auto kernel = scan_lookback_kernel<T, Op, ROWS, INCLUSIVE, PREFETCH>;
        const size_t tiles = ceil_div(c.n, tile_elems(ROWS));
        const size_t xentries = ceil_div(tiles, kWindow) * kWindow;   // transposed second-level array, 64 rows
        if (desc_bytes(tiles) + desc_bytes(xentries) > c.temp_bytes) return KS_ERR_WORKSPACE;
        static int per_cu = 0;   // resident workgroups per compute unit for this variant, as verified below
        if (per_cu == 0) {
            int nb = 0;
            hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, kBlock, 0);
            if (e != hipSuccess) return set_hip_error(e);
            // The query is an upper bound only; run the kernel in its residency-check mode and
            // step down until every workgroup of the grid is seen running at once.  One-off per
            // variant and device; it synchronises the stream.
            int verified = 0;
            for (int tryb = nb; tryb >= 1 && !verified; --tryb) {
                uint32_t zero[2] = {0u, 0u};
                e = hipMemcpyAsync(c.dev->residency, zero, sizeof(zero), hipMemcpyHostToDevice, c.stream);
                if (e != hipSuccess) return set_hip_error(e);
                hipLaunchKernelGGL(kernel, dim3((unsigned)(tryb * c.dev->cus)), dim3(kBlock), 0, c.stream,
                                   static_cast<const T *>(nullptr), static_cast<T *>(nullptr), (size_t)0,
                                   static_cast<uint64_t *>(nullptr), static_cast<uint64_t *>(nullptr), 0u, 0u,
                                   (uint32_t)(1u << 16), c.dev->abort_flag, 0, c.dev->residency);
                if ((e = hipGetLastError()) != hipSuccess) return set_hip_error(e);
                uint32_t seen[2] = {0u, 1u};
                e = hipMemcpyAsync(seen, c.dev->residency, sizeof(seen), hipMemcpyDeviceToHost, c.stream);
                if (e != hipSuccess) return set_hip_error(e);
                if ((e = hipStreamSynchronize(c.stream)) != hipSuccess) return set_hip_error(e);
                if (seen[1] == 0u) verified = tryb;
            }
            if (verified < 1) return KS_ERR_WORKSPACE;
            per_cu = verified;
        }
        long long want = options().wgs_per_cu;
        int use = (want > 0 && want < per_cu) ? (int)want : per_cu;
        size_t grid = (size_t)use * (size_t)c.dev->cus;
        if (options().grid_mode == 1 || grid > tiles) grid = tiles;
        options().last_grid = (long long)grid;
        options().last_resident_per_cu = per_cu;
        uint64_t *desc = static_cast<uint64_t *>(c.temp);
        uint64_t *xdesc = desc + desc_bytes(tiles) / sizeof(uint64_t);
        if (c.clear_descriptors) {
            const size_t words = (desc_bytes(tiles) + desc_bytes(xentries)) / sizeof(uint64_t);
            const unsigned fb = (unsigned)(ceil_div(words, 256) < 1024 ? ceil_div(words, 256) : 1024);
            hipLaunchKernelGGL((fill_zero_kernel<0>), dim3(fb), dim3(256), 0, c.stream, desc, words);
        }
        long long spin = options().spin_limit;
        if (spin < 0) spin = 0;
        if (spin > 0xffffffffll) spin = 0xffffffffll;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kBlock), 0, c.stream, static_cast<const T *>(c.in),
                           static_cast<T *>(c.out), c.n, desc, xdesc, c.epoch, (uint32_t)tiles, (uint32_t)spin,
                           c.dev->abort_flag, aligned, static_cast<uint32_t *>(nullptr));
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? KS_OK : set_hip_error(e);
    }

    template <int ROWS>
    static int lookback_rows_dispatch(const ScanCall &c, int aligned) {
        const bool pf = lookback_prefetch();
        if (c.inclusive)
            return pf ? launch_lookback<ROWS, true, true>(c, aligned) : launch_lookback<ROWS, true, false>(c, aligned);
        return pf ? launch_lookback<ROWS, false, true>(c, aligned) : launch_lookback<ROWS, false, false>(c, aligned);
    }

    static int run_lookback(const ScanCall &c, int aligned) {
        switch (lookback_rows()) {
            case 2: return lookback_rows_dispatch<2>(c, aligned);
            case 4: return lookback_rows_dispatch<4>(c, aligned);
            case 16: return lookback_rows_dispatch<16>(c, aligned);
            default: return lookback_rows_dispatch<8>(c, aligned);
        }
    }

    // ---- reduce-then-scan ----------------------------------------------------
    static int launch_tile_scan(bool inclusive, const T *in, T *out, size_t n, const A *seeds, int aligned,
                                hipStream_t s) {
        const size_t tiles = ceil_div(n, tile_elems(kRtsRows));
        if (inclusive)
            hipLaunchKernelGGL((tile_scan_kernel<T, Op, kRtsRows, true>), dim3((unsigned)tiles), dim3(kBlock), 0, s, in,
                               out, n, seeds, aligned);
        else
            hipLaunchKernelGGL((tile_scan_kernel<T, Op, kRtsRows, false>), dim3((unsigned)tiles), dim3(kBlock), 0, s,
                               in, out, n, seeds, aligned);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? KS_OK : set_hip_error(e);
    }

    static int run_rts(bool inclusive, const T *in, T *out, size_t n, int aligned, char *temp, size_t temp_bytes,
                       hipStream_t s) {
        const size_t tile = tile_elems(kRtsRows);
        const size_t tiles = ceil_div(n, tile);
        if (tiles <= 1) return launch_tile_scan(inclusive, in, out, n, nullptr, aligned, s);
        const size_t need = align_up(tiles * sizeof(A), 256);
        if (need > temp_bytes) return KS_ERR_WORKSPACE;
        A *agg = reinterpret_cast<A *>(temp);
        hipLaunchKernelGGL((tile_reduce_kernel<T, Op, kRtsRows>), dim3((unsigned)tiles), dim3(kBlock), 0, s, in, n, agg,
                           aligned);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return set_hip_error(e);
        // aggregates -> exclusive prefixes of the tiles, in place (scratch is 256-byte aligned)
        int st = Pair<A, Op>::run_rts(false, agg, agg, tiles, 1, temp + need, temp_bytes - need, s);
        if (st != KS_OK) return st;
        return launch_tile_scan(inclusive, in, out, n, agg, aligned, s);
    }

    static int run(const ScanCall &c) {
        const int aligned = (((uintptr_t)c.in | (uintptr_t)c.out) & 15u) == 0 ? 1 : 0;
        if (c.algo == KS_ALGO_LOOKBACK) return run_lookback(c, aligned);
        return run_rts(c.inclusive != 0, static_cast<const T *>(c.in), static_cast<T *>(c.out), c.n, aligned,
                       static_cast<char *>(c.temp), c.temp_bytes, c.stream);
    }

    static const PairEntry *entry() {
        static const PairEntry e = {sizeof(T), alignof(T), &Pair::temp_bytes, &Pair::pick_algo, &Pair::run};
        return &e;
    }
};

}  // namespace ks
