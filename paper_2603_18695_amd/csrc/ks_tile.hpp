// Tile-level pieces of the scan: coalesced 16-byte global access, the scan of a
// thread's items in registers, and the per-wave combination (paper Sec. V-B,
// second paragraph; Sec. IV-C for the wide loads and the items-per-thread idea).
//
// Register arrangement.  A workgroup of WAVES wave64s owns one tile.  Wave w
// owns a contiguous run of 64*ROWS granules of 16 bytes; inside it, "row" j is
// 64 consecutive granules and lane l holds granule l of every row.  Each global
// access instruction of a wave therefore touches 1 KiB of consecutive bytes.
// Element order inside a wave is (row, lane, position in granule), so the scan
// is: fold inside each granule, one wave scan per row over the granule totals,
// then a short serial chain over the ROWS row totals.  Operand order is kept at
// every level, so non-commutative operators are safe.
//
// IO is the element type in memory, A = Op::acc the type held in registers.
#pragma once

#include "ks_wave.hpp"

namespace ks {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <class IO, int ROWS_>
struct TileShape {
    static_assert(sizeof(IO) == 4 || sizeof(IO) == 8 || sizeof(IO) == 16, "element must be 4, 8 or 16 bytes");
    static constexpr int ROWS = ROWS_;
    static constexpr int G = 16 / (int)sizeof(IO);  // elements per 16-byte granule
    static constexpr int ITEMS = ROWS * G;          // elements per thread
    static constexpr int WAVE_ELEMS = kWave * ITEMS;
};

template <class IO, int G>
struct Granule {
    IO e[G];
};

// Items of one thread: x[j][k] = element k of the lane's granule in row j.
template <class A, int ROWS, int G>
struct ThreadItems {
    A x[ROWS][G];
};

// The lane's granules as they come from memory, before conversion to the
// accumulation type.  A prefetched tile is parked in this form: it costs
// 4 registers per row whatever the accumulator's size.
template <int ROWS>
struct RawItems {
    u32x4 v[ROWS];
};

// Load the lane's granules.  `first` = index of the first element of the lane's
// row-0 granule.  vec: every granule is inside [0, n) and 16-byte aligned.
// Otherwise element-wise, elements at or past n read as the identity.
template <class IO, int ROWS, class Op>
__device__ __forceinline__ void load_raw(const IO *__restrict__ in, size_t first, size_t n, bool vec,
                                         RawItems<ROWS> &raw) {
    constexpr int G = TileShape<IO, ROWS>::G;
    if (vec) {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const u32x4 *p = reinterpret_cast<const u32x4 *>(in + first + (size_t)j * kWave * G);
            raw.v[j] = __builtin_nontemporal_load(p);
        }
    } else {
        const IO fill = convert<IO>(Op::identity());
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            Granule<IO, G> g;
#pragma unroll
            for (int k = 0; k < G; ++k) {
                // unconditional in-bounds load, then a select on the value (a select between the
                // two addresses would put `fill` in scratch memory)
                const size_t i = first + (size_t)j * kWave * G + k;
                const IO v = in[i < n ? i : 0];
                g.e[k] = (i < n) ? v : fill;
            }
            raw.v[j] = __builtin_bit_cast(u32x4, g);
        }
    }
}

template <class IO, int ROWS, class Op>
__device__ __forceinline__ void unpack_items(const RawItems<ROWS> &raw,
                                             ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    using A = typename Op::acc;
    constexpr int G = TileShape<IO, ROWS>::G;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        Granule<IO, G> g = __builtin_bit_cast(Granule<IO, G>, raw.v[j]);
#pragma unroll
        for (int k = 0; k < G; ++k) it.x[j][k] = convert<A>(g.e[k]);
    }
}

template <class IO, int ROWS, class Op>
__device__ __forceinline__ void load_items(const IO *__restrict__ in, size_t first, size_t n, bool vec,
                                           ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    RawItems<ROWS> raw;
    load_raw<IO, ROWS, Op>(in, first, n, vec, raw);
    unpack_items<IO, ROWS, Op>(raw, it);
}

template <class IO, int ROWS, class A>
__device__ __forceinline__ void store_items(IO *__restrict__ out, size_t first, size_t n, bool vec,
                                            const ThreadItems<A, ROWS, TileShape<IO, ROWS>::G> &it) {
    constexpr int G = TileShape<IO, ROWS>::G;
    if (vec) {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            Granule<IO, G> g;
#pragma unroll
            for (int k = 0; k < G; ++k) g.e[k] = convert<IO>(it.x[j][k]);
            u32x4 *p = reinterpret_cast<u32x4 *>(out + first + (size_t)j * kWave * G);
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, g), p);
        }
    } else {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
#pragma unroll
            for (int k = 0; k < G; ++k) {
                size_t i = first + (size_t)j * kWave * G + k;
                if (i < n) out[i] = convert<IO>(it.x[j][k]);
            }
        }
    }
}

// Result of scanning one wave's run in registers.
template <class A, int ROWS>
struct WaveScan {
    A lane_base[ROWS];   // combination of everything in the wave's run before the lane's granule in row j
    A wave_total;        // combination of the whole run (same in every lane)
};

// In place: it.x[j][k] becomes the inclusive fold of the lane's granule up to k.
template <class A, int ROWS, int G, class Op>
__device__ __forceinline__ WaveScan<A, ROWS> scan_wave_run(ThreadItems<A, ROWS, G> &it, Op op) {
    WaveScan<A, ROWS> r;
    A inc[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
#pragma unroll
        for (int k = 1; k < G; ++k) it.x[j][k] = op(it.x[j][k - 1], it.x[j][k]);
        inc[j] = it.x[j][G - 1];
    }
#pragma unroll
    for (int j = 0; j < ROWS; ++j) inc[j] = wave_inclusive_scan(inc[j], op);
    A carry = Op::identity();   // rows before row j
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        A before_lane = wave_shift_up(inc[j], Op::identity());
        r.lane_base[j] = op(carry, before_lane);
        carry = op(carry, read_lane(inc[j], kWave - 1));
    }
    r.wave_total = carry;
    return r;
}

// Turn the thread's items into final outputs given `prefix` = combination of
// everything before this wave's run (tile prefix and earlier waves).
template <bool INCLUSIVE, class A, int ROWS, int G, class Op>
__device__ __forceinline__ void apply_prefix(ThreadItems<A, ROWS, G> &it, const WaveScan<A, ROWS> &ws,
                                             const A &prefix, Op op) {
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const A base = op(prefix, ws.lane_base[j]);
        if (INCLUSIVE) {
#pragma unroll
            for (int k = 0; k < G; ++k) it.x[j][k] = op(base, it.x[j][k]);
        } else {
#pragma unroll
            for (int k = G - 1; k >= 1; --k) it.x[j][k] = op(base, it.x[j][k - 1]);
            it.x[j][0] = base;
        }
    }
}

}  // namespace ks
