// Tile-level pieces of the scan: coalesced 16-byte buffer access, the scan of a
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

// One tile of `in` or `out` seen through a buffer resource: base = first element
// of the tile, extent = the tile's valid bytes.  The hardware range-checks every
// dword of a buffer access against the extent: reads past it return zero and
// writes past it are dropped, so the ragged last tile and pointers that are only
// element-aligned go through the same 16-byte instructions as everything else
// (the paper's Sec. IV-D decomposes misaligned accesses in software instead).
struct TileWindow {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t valid_bytes;
};

template <class IO>
__device__ __forceinline__ TileWindow tile_window(const IO *base, size_t n, size_t tile_first, size_t tile_elems) {
    const size_t left = n > tile_first ? n - tile_first : 0;
    const uint32_t valid = (uint32_t)((left < tile_elems ? left : tile_elems) * sizeof(IO));
    TileWindow w;
    // raw buffer (stride 0), 32-bit data format, no swizzle: the gfx90a / gfx94x / gfx950 encoding
    w.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<IO *>(base + tile_first), 0, (int)valid, 0x00020000);
    w.valid_bytes = valid;
    return w;
}

constexpr int kNonTemporal = 2;   // "nt" bit of the buffer instructions' cache policy

// Load the lane's granules.  lane_bytes = byte offset of the lane's row-0 granule
// inside the tile; rows are 1 KiB apart.  (Signed arithmetic on purpose: it lets the
// compiler put the row offset into the instruction's immediate field, so that
// four rows share one address register.)
template <int ROWS>
__device__ __forceinline__ void load_raw(const TileWindow &w, int lane_bytes, RawItems<ROWS> &raw) {
#pragma unroll
    for (int j = 0; j < ROWS; ++j)
        raw.v[j] = __builtin_amdgcn_raw_buffer_load_b128(w.rsrc, lane_bytes + j * (kWave * 16), 0, kNonTemporal);
}

// Raw granules -> accumulation type.  In a partial tile the elements past the
// end (read as zero by the hardware) become the operator's identity.
template <class IO, int ROWS, class Op>
__device__ __forceinline__ void unpack_items(const RawItems<ROWS> &raw, int lane_bytes, uint32_t valid_bytes,
                                             bool partial,
                                             ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    using A = typename Op::acc;
    constexpr int G = TileShape<IO, ROWS>::G;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        Granule<IO, G> g = __builtin_bit_cast(Granule<IO, G>, raw.v[j]);
#pragma unroll
        for (int k = 0; k < G; ++k) it.x[j][k] = convert<A>(g.e[k]);
    }
    if (partial) {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const int at = lane_bytes + j * (kWave * 16) + k * (int)sizeof(IO);
                if ((uint32_t)at >= valid_bytes) it.x[j][k] = Op::identity();
            }
        }
    }
}

template <class IO, int ROWS, class Op>
__device__ __forceinline__ void load_items(const TileWindow &w, int lane_bytes, bool partial,
                                           ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    RawItems<ROWS> raw;
    load_raw<ROWS>(w, lane_bytes, raw);
    unpack_items<IO, ROWS, Op>(raw, lane_bytes, w.valid_bytes, partial, it);
}

template <class IO, int ROWS, class A>
__device__ __forceinline__ void store_items(const TileWindow &w, int lane_bytes,
                                            const ThreadItems<A, ROWS, TileShape<IO, ROWS>::G> &it) {
    constexpr int G = TileShape<IO, ROWS>::G;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        Granule<IO, G> g;
#pragma unroll
        for (int k = 0; k < G; ++k) g.e[k] = convert<IO>(it.x[j][k]);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, g), w.rsrc,
                                               lane_bytes + j * (kWave * 16), 0, kNonTemporal);
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
