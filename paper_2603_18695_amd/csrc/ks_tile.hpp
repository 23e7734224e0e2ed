// Tile-level pieces of the scan: coalesced 16-byte buffer access, the scan of a
// thread's items in registers, and the per-wave combination (paper Sec. V-B,
// second paragraph; Sec. IV-C for the wide loads and the items-per-thread idea).
//
// Striped register arrangement (first part of the file).  A workgroup owns one
// tile; each of its data waves owns a contiguous run of 64*ROWS granules of 16
// bytes; inside it, "row" j is 64 consecutive granules and lane l holds granule
// l of every row.  Each global access instruction of a wave therefore touches
// 1 KiB of consecutive bytes.  Element order inside a wave is (row, lane,
// position in granule), so the scan is: fold inside each granule, one wave scan
// per row over the granule totals, then a short serial chain over the ROWS row
// totals.  Operand order is kept at every level, so non-commutative operators
// are safe.  The blocked arrangement (second part) keeps the striped global
// accesses and exchanges the granules through LDS so that a lane holds ROWS
// consecutive granules; strided views (last part) access single elements.
//
// IO is the element type in memory, A = Op::acc the type held in registers.
#pragma once

#include "ks_wave.hpp"

namespace ks {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Element sizes that fit a 16-byte granule a whole number of times run in every arrangement;
// the others only in the blocked one (BlockedShape, below).
template <class IO>
constexpr bool granule_sized() { return sizeof(IO) == 2 || sizeof(IO) == 4 || sizeof(IO) == 8 || sizeof(IO) == 16; }

template <class IO, int ROWS_>
struct TileShape {
    static_assert(16 % sizeof(IO) == 0, "a 16-byte granule must hold whole elements in the striped arrangement");
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
    // Elements narrower than a dword: the range check works on dwords, so the extent is rounded up
    // to the dword that holds the last element; `base` is dword-aligned there, the surplus bytes
    // lie in the same dword, and valid_bytes stays exact.  Loads mask what they read past
    // valid_bytes; stores write the granule that holds such a dword element by element
    // (apply_prefix_and_store).
    const uint32_t extent = sizeof(IO) < 4 ? (valid + 3u) & ~3u : valid;
    // raw buffer (stride 0), 32-bit data format, no swizzle: the gfx90a / gfx94x / gfx950 encoding
    w.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<IO *>(base + tile_first), 0, (int)extent, 0x00020000);
    w.valid_bytes = valid;
    return w;
}

constexpr int kNonTemporal = 2;   // "nt" bit of the buffer instructions' cache policy

// The row offsets (multiples of 1 KiB) fit the buffer instructions' 12-bit
// immediate field four rows at a time, but only if the additions are still next
// to the instruction when it is selected: inside the tile loop the compiler
// would hoist them and keep one address register per row.  With PIN the offset
// passes through an empty asm statement, which pins the additions to the loop
// body and saves those registers; callers that have registers to spare leave
// it off (the register allocation and the waits the compiler derives from it
// change with it, and the 4-byte kernels measured 8 % slower with it).  (Signed
// arithmetic on purpose: unsigned offsets are not folded into the immediate.)
template <bool PIN>
__device__ __forceinline__ int pinned(int lane_bytes) {
    if (PIN) asm volatile("" : "+v"(lane_bytes));
    return lane_bytes;
}

// Load the lane's granules.  lane_bytes = byte offset of the lane's row-0 granule
// inside the tile; rows are 1 KiB apart.
template <int ROWS, bool PIN>
__device__ __forceinline__ void load_raw(const TileWindow &w, int lane_bytes, RawItems<ROWS> &raw) {
    const int at = pinned<PIN>(lane_bytes);
#pragma unroll
    for (int j = 0; j < ROWS; ++j)
        raw.v[j] = __builtin_amdgcn_raw_buffer_load_b128(w.rsrc, at + j * (kWave * 16), 0, kNonTemporal);
}

// Raw granules -> accumulation type, through the operator's map if it has one
// (scan(f, op, src), paper Sec. IV-A).  In a partial tile the elements past the
// end (read as zero by the hardware) become the operator's identity.
template <class IO, int ROWS, class Op, bool PIN>
__device__ __forceinline__ void unpack_items(const RawItems<ROWS> &raw, int lane_bytes, uint32_t valid_bytes,
                                             bool partial,
                                             ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    using A = typename Op::acc;
    constexpr int G = TileShape<IO, ROWS>::G;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        Granule<IO, G> g = __builtin_bit_cast(Granule<IO, G>, raw.v[j]);
#pragma unroll
        for (int k = 0; k < G; ++k) it.x[j][k] = convert<A>(typename MapOf<Op>::type()(g.e[k]));
    }
    if (partial) {
        const int at0 = pinned<PIN>(lane_bytes);   // keeps the element offsets out of the registers of full tiles
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const int at = at0 + j * (kWave * 16) + k * (int)sizeof(IO);
                if ((uint32_t)at >= valid_bytes) it.x[j][k] = Op::identity();
            }
        }
    }
}

template <class IO, int ROWS, class Op, bool PIN>
__device__ __forceinline__ void load_items(const TileWindow &w, int lane_bytes, bool partial,
                                           ThreadItems<typename Op::acc, ROWS, TileShape<IO, ROWS>::G> &it) {
    RawItems<ROWS> raw;
    load_raw<ROWS, PIN>(w, lane_bytes, raw);
    unpack_items<IO, ROWS, Op, PIN>(raw, lane_bytes, w.valid_bytes, partial, it);
}

// First half of the scan of one wave's run: what the rest of the workgroup is
// waiting for.  In place, it.x[j][k] becomes the inclusive fold of the lane's
// granule up to k; lane_base[j] = combination of everything in the run before
// the lane's granule in row j; wave_total = combination of the whole run (the
// same value in every lane).  The items themselves are finished by
// finish_wave_run, after the total has been handed on: how soon a tile's
// aggregate is published decides how long other tiles wait for it.
template <class A, int ROWS>
struct WaveScan {
    A lane_base[ROWS];
    A wave_total;
};

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
    for (int j = 0; j < ROWS; ++j) inc[j] = wave_inclusive_scan(inc[j], op);   // granule totals, lanes 0..l
    A carry = Op::identity();   // rows before row j
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const A before_lane = wave_shift_up(inc[j], Op::identity());
        r.lane_base[j] = op(carry, before_lane);
        carry = op(carry, read_lane(inc[j], kWave - 1));
    }
    r.wave_total = carry;
    return r;
}

// Second half: it.x[j][k] becomes the scan of the wave's run alone, inclusive
// or exclusive (the very first element of the run then becomes the identity).
// After this only the items stay in registers: what comes from outside the run
// (earlier waves, earlier tiles) is one value that apply_prefix_and_store puts
// in front of every item.
template <bool INCLUSIVE, class A, int ROWS, int G, class Op>
__device__ __forceinline__ void finish_wave_run(ThreadItems<A, ROWS, G> &it, const WaveScan<A, ROWS> &ws, Op op) {
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const A base = ws.lane_base[j];
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

// Combination of a whole wave's run for a COMMUTATIVE operator, by the shortest
// route: every lane folds its own items, one wave reduction.  The time from the
// arrival of a tile to the publication of its aggregate is on the critical path
// of the whole scan (the next tile is only requested once the totals are out,
// and other tiles wait for the aggregate), so the separate-loop forms take this
// route first and scan afterwards, while the look-back wave is busy.  The value
// can differ from the scan's own total in the last bits for floating point (a
// different association); every output is still a valid association of its
// prefix.  Items are not modified.
template <class A, int ROWS, int G, class Op>
__device__ __forceinline__ A reduce_wave_run_any_order(const ThreadItems<A, ROWS, G> &it, Op op) {
    static_assert(Op::commutative, "order-free reduction needs a commutative operator");
    A mine = it.x[0][0];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
#pragma unroll
        for (int k = 0; k < G; ++k)
            if (j != 0 || k != 0) mine = op(mine, it.x[j][k]);
    }
    return read_lane(wave_inclusive_scan(mine, op), kWave - 1);
}

// Both halves in one pass, row by row, for callers that do not need the wave
// total before the items are finished: no lane_base array is kept, which for
// one-element granules (16-byte types) saves as many registers as the tile
// itself takes.  Returns the combination of the whole run.
template <bool INCLUSIVE, class A, int ROWS, int G, class Op>
__device__ __forceinline__ A scan_wave_run_in_place(ThreadItems<A, ROWS, G> &it, Op op) {
    A carry = Op::identity();   // rows before row j
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
#pragma unroll
        for (int k = 1; k < G; ++k) it.x[j][k] = op(it.x[j][k - 1], it.x[j][k]);
        const A inc = wave_inclusive_scan(it.x[j][G - 1], op);   // granule totals, lanes 0..l
        if (INCLUSIVE && G == 1) {
            it.x[j][0] = (j == 0) ? inc : op(carry, inc);
        } else {
            const A before_lane = wave_shift_up(inc, Op::identity());
            const A base = (j == 0) ? before_lane : op(carry, before_lane);
            if (INCLUSIVE) {
#pragma unroll
                for (int k = 0; k < G; ++k) it.x[j][k] = op(base, it.x[j][k]);
            } else {
#pragma unroll
                for (int k = G - 1; k >= 1; --k) it.x[j][k] = op(base, it.x[j][k - 1]);
                it.x[j][0] = base;
            }
        }
        const A row_total = read_lane(inc, kWave - 1);
        carry = (j == 0) ? row_total : op(carry, row_total);
    }
    return carry;
}

// Final outputs: `prefix` (combination of everything before this wave's run)
// in front of every item, converted to the memory type and stored.
template <class IO, int ROWS, class A, class Op, bool PIN>
__device__ __forceinline__ void apply_prefix_and_store(const TileWindow &w, int lane_bytes,
                                                       const ThreadItems<A, ROWS, TileShape<IO, ROWS>::G> &it,
                                                       const A &prefix, Op op) {
    constexpr int G = TileShape<IO, ROWS>::G;
    const int at = pinned<PIN>(lane_bytes);
    // 2-byte elements: an array of odd length ends in the middle of a dword, and the other half of
    // that dword is not the caller's to write.  Only then (one tile per call at most) the granule
    // that holds it goes out element by element; a 16-byte store would write the whole dword.
    const bool ragged_dword = sizeof(IO) < 4 && (w.valid_bytes & 3u) != 0;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        Granule<IO, G> g;
#pragma unroll
        for (int k = 0; k < G; ++k) g.e[k] = convert<IO>(op(prefix, it.x[j][k]));
        if constexpr (sizeof(IO) == 2) {
            const uint32_t first = (uint32_t)(at + j * (kWave * 16));
            if (ragged_dword && first < w.valid_bytes && first + 16u > (w.valid_bytes & ~3u)) {
#pragma unroll
                for (int k = 0; k < G; ++k) {
                    if (first + (uint32_t)k * 2u < w.valid_bytes)
                        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, g.e[k]), w.rsrc,
                                                              (int)first + k * 2, 0, kNonTemporal);
                }
                continue;
            }
        }
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, g), w.rsrc, at + j * (kWave * 16), 0,
                                               kNonTemporal);
    }
}

// ---------------------------------------------------------------------------
// Blocked arrangement.  The striped arrangement above costs one 64-lane scan per
// row: about 90 vector instructions per KiB for a 16-byte element, half a tile
// period at full memory rate.  Here each wave passes its granules through a
// private LDS region so that lane l ends up with ROWS CONSECUTIVE granules of
// the run (global accesses stay striped and coalesced, paper Sec. IV-C; the
// exchange replaces the shuffles of Sec. IV-A by LDS).  Element order inside a
// wave is then (lane, granule, position): a serial scan in registers and ONE
// 64-lane scan of the lane totals per tile.
//
// LDS layout of a wave's region, in 16-byte slots: granule g of the run (g =
// row * 64 + lane in the striped view, g = lane * ROWS + i in the blocked view)
// sits at slot (g / ROWS) * STRIDE + g % ROWS with STRIDE = ROWS | 1: an odd
// lane stride keeps the blocked 16-byte accesses of 16 neighbouring lanes on
// distinct banks.  A wave's LDS instructions execute in order, and the wait
// between the two phases makes that explicit; no other wave touches the region,
// so no barrier is needed.
// ---------------------------------------------------------------------------
template <int ROWS>
struct Stage {
    static constexpr int STRIDE = ROWS | 1;
    static constexpr int SLOTS = kWave * STRIDE;   // per wave
};

constexpr int kWaitLds = 0xC07F;   // s_waitcnt lgkmcnt(0), other counters untouched (gfx9 encoding)

template <int ROWS>
__device__ __forceinline__ int stage_slot_of_striped(int row, int lane) {
    const int g = row * kWave + lane;
    return (g / ROWS) * Stage<ROWS>::STRIDE + g % ROWS;
}

// Striped view in registers -> the wave's LDS region ...
template <int ROWS>
__device__ __forceinline__ void stage_striped(u32x4 *region, const RawItems<ROWS> &striped) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int j = 0; j < ROWS; ++j) region[stage_slot_of_striped<ROWS>(j, lane)] = striped.v[j];
}

// ... and back out as the blocked view.
template <int ROWS>
__device__ __forceinline__ void fetch_blocked(const u32x4 *region, RawItems<ROWS> &blocked) {
    const int lane = threadIdx.x & (kWave - 1);
    __builtin_amdgcn_s_waitcnt(kWaitLds);
#pragma unroll
    for (int i = 0; i < ROWS; ++i) blocked.v[i] = region[lane * Stage<ROWS>::STRIDE + i];
}

// Registers hold the striped view on entry and the blocked view on return.
template <int ROWS>
__device__ __forceinline__ void striped_to_blocked(u32x4 *region, RawItems<ROWS> &r) {
    stage_striped<ROWS>(region, r);
    fetch_blocked<ROWS>(region, r);
}

template <int ROWS>
__device__ __forceinline__ void blocked_to_striped(u32x4 *region, RawItems<ROWS> &r) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int i = 0; i < ROWS; ++i) region[lane * Stage<ROWS>::STRIDE + i] = r.v[i];
    __builtin_amdgcn_s_waitcnt(kWaitLds);
#pragma unroll
    for (int j = 0; j < ROWS; ++j) r.v[j] = region[stage_slot_of_striped<ROWS>(j, lane)];
}

// In the blocked view a lane holds ROWS consecutive granules, i.e. ROWS * 16 consecutive bytes of
// the wave's run: E whole elements of any size that divides that (ROWS = 8: 128 bytes, ROWS = 9:
// 144 bytes).  This is what serves elements that are not 4, 8 or 16 bytes: the global accesses
// stay 16-byte granules whatever the element (paper Sec. IV-A: composite types of any size).
template <class IO, int ROWS>
struct BlockedShape {
    static_assert((ROWS * 16) % sizeof(IO) == 0, "the element size must divide the lane's ROWS * 16 bytes");
    static constexpr int E = ROWS * 16 / (int)sizeof(IO);   // elements per lane
    static constexpr int WAVE_ELEMS = kWave * E;
};
template <class IO, int ROWS>
constexpr bool blocked_fits() { return (ROWS * 16) % sizeof(IO) == 0; }

// Items of one lane in the blocked view: y[k] = the lane's k-th consecutive element.
template <class A, int E>
struct LaneItems {
    A y[E];
};
template <class IO, int E>
struct LaneChunk {
    IO e[E];
};

// Blocked raw granules -> accumulation type.  run_bytes = byte offset of the wave's run inside
// the tile (for the identity fix-up of a partial tile).
template <class IO, int ROWS, class Op>
__device__ __forceinline__ void unpack_blocked(const RawItems<ROWS> &raw, int run_bytes, uint32_t valid_bytes, bool partial,
                                               LaneItems<typename Op::acc, BlockedShape<IO, ROWS>::E> &it) {
    using A = typename Op::acc;
    constexpr int E = BlockedShape<IO, ROWS>::E;
    const LaneChunk<IO, E> c = __builtin_bit_cast(LaneChunk<IO, E>, raw);
#pragma unroll
    for (int k = 0; k < E; ++k) it.y[k] = convert<A>(typename MapOf<Op>::type()(c.e[k]));
    if (partial) {
        const int lane = threadIdx.x & (kWave - 1);
        const int at0 = pinned<true>(run_bytes + lane * (ROWS * 16));
#pragma unroll
        for (int k = 0; k < E; ++k) {
            if ((uint32_t)(at0 + k * (int)sizeof(IO)) >= valid_bytes) it.y[k] = Op::identity();
        }
    }
}

// Serial inclusive scan of the lane's E consecutive elements, then one wave scan of the lane
// totals.  Returns the combination of the whole run; lane_before = combination of the lanes
// before this one.
template <class A, int E, class Op>
__device__ __forceinline__ A scan_blocked_run(LaneItems<A, E> &it, A &lane_before, Op op) {
#pragma unroll
    for (int k = 1; k < E; ++k) it.y[k] = op(it.y[k - 1], it.y[k]);
    const A upto = wave_inclusive_scan(it.y[E - 1], op);
    lane_before = wave_shift_up(upto, Op::identity());
    return read_lane(upto, kWave - 1);
}

// Final outputs of the blocked view as raw granules: `before` (everything before this lane's
// first element) in front of every item, shifted by one element for the exclusive scan.
template <bool INCLUSIVE, class IO, int ROWS, class A, class Op>
__device__ __forceinline__ void apply_blocked(const LaneItems<A, BlockedShape<IO, ROWS>::E> &it, const A &before, Op op,
                                              RawItems<ROWS> &out) {
    constexpr int E = BlockedShape<IO, ROWS>::E;
    LaneChunk<IO, E> c;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        if (INCLUSIVE)
            c.e[k] = convert<IO>(op(before, it.y[k]));
        else if (k == 0)
            c.e[k] = convert<IO>(before);
        else
            c.e[k] = convert<IO>(op(before, it.y[k - 1]));
    }
    out = __builtin_bit_cast(RawItems<ROWS>, c);
}

template <int ROWS, bool PIN>
__device__ __forceinline__ void store_raw(const TileWindow &w, int lane_bytes, const RawItems<ROWS> &raw) {
    const int at = pinned<PIN>(lane_bytes);
#pragma unroll
    for (int j = 0; j < ROWS; ++j)
        __builtin_amdgcn_raw_buffer_store_b128(raw.v[j], w.rsrc, at + j * (kWave * 16), 0, kNonTemporal);
}

// ---------------------------------------------------------------------------
// Strided views (paper Sec. IV-C: the element-wise fallback for data that is not
// contiguous keeps the items-per-thread structure).  Element i of the view lives
// at base[i * stride]; accesses are one element wide and the register arrangement
// is the striped one with one-element granules (G = 1: lane l of row j holds
// element j * 64 + l of the wave's run), so that the lanes of one access are
// neighbours in the view and share cache lines as far as the stride allows.
// ---------------------------------------------------------------------------
template <class IO, int ROWS, class Op>
__device__ __forceinline__ void load_items_strided(const IO *base, size_t stride, size_t n, size_t run_first,
                                                   ThreadItems<typename Op::acc, ROWS, 1> &it) {
    using A = typename Op::acc;
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const size_t i = run_first + (size_t)j * kWave + lane;
        it.x[j][0] = i < n ? convert<A>(typename MapOf<Op>::type()(base[i * stride])) : Op::identity();
    }
}

template <class IO, int ROWS, class A, class Op>
__device__ __forceinline__ void apply_prefix_and_store_strided(IO *base, size_t stride, size_t n, size_t run_first,
                                                               const ThreadItems<A, ROWS, 1> &it, const A &prefix,
                                                               Op op) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const size_t i = run_first + (size_t)j * kWave + lane;
        if (i < n) base[i * stride] = convert<IO>(op(prefix, it.x[j][0]));
    }
}

}  // namespace ks
