// Kernels of the scan library.
//
//   scan_lookback_kernel   single pass, decoupled look-back (paper Sec. V-B)
//   tile_reduce_kernel     reduce-then-scan, first kernel: one aggregate per tile
//   tile_scan_kernel       reduce-then-scan, last kernel: scan a tile from a seed
//   scan_lookback_strided_kernel  the look-back scan over strided views (paper Sec. IV-C)
//   fill_zero_kernel       clears scratch whose contents are unknown
//   copy_kernel            vectorised copy, the bandwidth ceiling (paper Sec. IV-C)
// (mapreduce_kernel, the single-launch reduction of Sec. V-A, is in ks_reduce.hpp.)
//
// Tile descriptors (paper Sec. V-B: per-tile aggregate, inclusive prefix and a
// partial / prefix status flag; Sec. IV-B for the hazard the flag guards).  The
// paper stores value and flag separately and orders them with a release store
// and an acquire load, which on this GPU means writing back and invalidating a
// per-XCD L2.  Here every 32-bit word of the value travels in one 64-bit word
// together with its status tag, written and read with relaxed device-scope
// atomics: a reader can never see a tag without the value it belongs to, so no
// fence, write-back or invalidate is needed.  A value of W words uses W tagged
// words and is accepted only when all W tags agree.  The tag also carries a
// call epoch, so descriptors left by earlier calls read as "not set" and the
// array never has to be cleared between calls.
#pragma once

#include "ks_tile.hpp"

namespace ks {

// Workgroup shapes: the reduce-then-scan kernels and the copy kernel use 4
// waves; the look-back kernel is compiled for 4, 8 and 16 waves, one of which
// does the look-back and the others the data.
constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

constexpr uint32_t kUnset = 0;
constexpr uint32_t kPartial = 1;   // value = aggregate of the tile alone
constexpr uint32_t kPrefix = 2;    // value = combination of tiles 0..t

__device__ __forceinline__ void desc_store_word(uint64_t *p, uint32_t tag, uint32_t payload) {
    __hip_atomic_store(p, ((uint64_t)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <class T>
__device__ __forceinline__ void desc_publish(uint64_t *desc, size_t entry, uint32_t epoch, uint32_t state,
                                             const T &value) {
    constexpr int W = WordsOf<T>::W;
    auto ws = to_words(value);
    uint64_t *p = desc + entry * W;
    const uint32_t tag = (epoch << 2) | state;
#pragma unroll
    for (int k = 0; k < W; ++k) desc_store_word(p + k, tag, ws.w[k]);
}

// Returns the state (kUnset if the descriptor is from another epoch or its
// words do not carry one common tag yet) and the value.
template <class T>
__device__ __forceinline__ uint32_t desc_read(const uint64_t *desc, size_t entry, uint32_t epoch, T &value) {
    constexpr int W = WordsOf<T>::W;
    const uint64_t *p = desc + entry * W;
    typename WordsOf<T>::type ws;
    uint32_t tag0 = 0;
    bool same = true;
#pragma unroll
    for (int k = 0; k < W; ++k) {
        uint64_t v = __hip_atomic_load(p + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t tag = (uint32_t)(v >> 32);
        ws.w[k] = (uint32_t)v;
        if (k == 0) tag0 = tag; else same = same && (tag == tag0);
    }
    value = from_words<T>(ws);
    if (!same || (tag0 >> 2) != epoch) return kUnset;
    return tag0 & 3u;
}

// Besides its own descriptor D(t) (PARTIAL: aggregate of tile t; PREFIX:
// combination of tiles 0..t) every tile has a second one, X(t):
//     PARTIAL  combination of the 64 tiles before t   (what t's first window gave)
//     PREFIX   combination of all tiles before t      (t's exclusive prefix)
// X is stored transposed, X(t) at [(t mod 64) * M + t / 64] with M = ceil(tiles/64),
// so that X(t-64), X(t-128), ..., X(t-4096) are 64 consecutive entries.  After a
// first window over D(t-64..t-1) a tile therefore covers 4096 more tiles with
// one coalesced 64-lane read, instead of walking back 64 tiles per memory round
// trip.  On this GPU a round trip takes 0.5 us idle and about 2 us while the
// memory system streams at full rate, and ~2000 tiles are in flight at once:
// the single-level walk of the paper (Sec. V-B) then advances the prefix more
// slowly than tiles arrive.  States, tags and the rule "nearest PREFIX ends the
// search, everything after it must be at least PARTIAL" are unchanged.
constexpr int kWindow = 64;

__device__ __forceinline__ size_t xdesc_index(uint32_t tile, uint32_t m) {
    return (size_t)(tile % kWindow) * m + tile / kWindow;
}

// Bookkeeping of the bounded wait: every failed poll of a look-back wave counts
// against `limit`.  A wave that gives up writes the call's sequence number (never
// zero) into the abort word of the call's stream; the other workgroups of the same
// call see it and stop as well, calls with another sequence number are not affected,
// and the host's status call reports and clears whatever it finds there.
struct SpinState {
    uint32_t spins;
    uint32_t limit;
    uint32_t *abort_flag;
    uint32_t call_seq;
};

__device__ __forceinline__ bool spin_once(SpinState &sp) {
    const int lane = threadIdx.x & (kWave - 1);
    ++sp.spins;
    if (sp.spins > sp.limit) {
        if (lane == 0) __hip_atomic_store(sp.abort_flag, sp.call_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    if ((sp.spins & 63u) == 0) {   // has another workgroup of this call given up?  (decided wave-uniformly)
        const uint32_t f = __hip_atomic_load(sp.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__ballot(f == sp.call_seq) != 0) return false;
    }
    __builtin_amdgcn_s_sleep(1);
    return true;
}

// One window: lane l owns entry base + first + l of `desc`, where first may be
// negative: entries before the start hold nothing (lane order = sequence order,
// lane 63 nearest).  Waits until the nearest PREFIX in the window and everything
// after it are visible, or, with no PREFIX in the window, until every lane is.
// On return `total` is the combination, in order, of the lanes from the nearest
// PREFIX on (all lanes if there is none) and found_prefix tells which.
template <class A, class Op>
__device__ __forceinline__ bool poll_window(const uint64_t *desc, size_t base, long long first, uint32_t epoch,
                                            SpinState &sp, A &total, bool &found_prefix) {
    const int lane = threadIdx.x & (kWave - 1);
    Op op;
    const long long mine = first + lane;
    A val = Op::identity();
    uint32_t st = (mine >= 0) ? kUnset : kPartial;   // nothing there: counts as an empty aggregate
    int top;
    for (;;) {
        if (st == kUnset) st = desc_read<A>(desc, base + (size_t)mine, epoch, val);
        const uint64_t prefix_mask = __ballot(st == kPrefix);
        const uint64_t unset_mask = __ballot(st == kUnset);
        top = prefix_mask ? 63 - __builtin_clzll(prefix_mask) : -1;
        const uint64_t needed = (top >= 63) ? 0ull : (~0ull << (top + 1));   // lanes after the nearest PREFIX
        if ((unset_mask & needed) == 0) break;
        if (!spin_once(sp)) return false;
    }
    if (lane < top) val = Op::identity();   // already covered by the PREFIX found
    total = read_lane(wave_inclusive_scan(val, op), kWave - 1);
    found_prefix = top >= 0;
    return true;
}

// Look-back executed by one full wave (paper Sec. V-B, third paragraph; window of
// 64 descriptors on wave64).  Returns false when the spin limit was hit or
// another workgroup gave up; otherwise exclusive_prefix = combination of all
// tiles before `tile`, and X(tile) has been published in state PREFIX.
template <class A, class Op>
__device__ __forceinline__ bool lookback(const uint64_t *desc, uint64_t *xdesc, uint32_t m, uint32_t tile,
                                         uint32_t epoch, uint32_t spin_limit, uint32_t *abort_flag, uint32_t call_seq,
                                         A &exclusive_prefix) {
    const int lane = threadIdx.x & (kWave - 1);
    Op op;
    SpinState sp{0u, spin_limit, abort_flag, call_seq};
    const size_t my_x = xdesc_index(tile, m);
    A running;
    bool done;
    // first window: D of the 64 tiles before this one
    if (!poll_window<A, Op>(desc, 0, (long long)tile - kWindow, epoch, sp, running, done)) return false;
    if (!done) {
        // tell later tiles what these 64 tiles add up to, then walk X(tile - 64), X(tile - 128), ...
        if (lane == 0) desc_publish<A>(xdesc, my_x, epoch, kPartial, running);
        const size_t row = (size_t)(tile % kWindow) * m;
        long long first = (long long)(tile / kWindow) - kWindow;   // window = entries first .. first+63 of the row
        while (!done) {
            A window;
            if (!poll_window<A, Op>(xdesc, row, first, epoch, sp, window, done)) return false;
            running = op(window, running);
            first -= kWindow;
        }
    }
    if (lane == 0) desc_publish<A>(xdesc, my_x, epoch, kPrefix, running);
    exclusive_prefix = running;
    return true;
}

// Cross-wave exchange through LDS (paper Sec. V-B: shared-memory exchange that
// yields the tile aggregate).  Returns the combination of the waves before
// this one; `aggregate` receives the whole tile's.  Wave totals are of the
// accumulation type; from here upwards everything is of the operator's chain type.
template <class Op, int WAVES>
__device__ __forceinline__ typename ChainOf<Op>::type exchange_wave_totals(
    typename WordsOf<typename Op::acc>::type *s_tot, const typename Op::acc &wave_total,
    typename ChainOf<Op>::type &aggregate) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    typename ChainOf<Op>::op cop;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    if (lane == 0) s_tot[wave] = to_words(wave_total);
    __syncthreads();
    C carry = ChainOf<Op>::op::identity();
    C all = ChainOf<Op>::op::identity();
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const C t = convert<C>(from_words<A>(s_tot[w]));
        if (w < wave) carry = cop(carry, t);
        all = cop(all, t);
    }
    aggregate = all;
    return carry;
}

// Byte offset, inside a tile, of the calling lane's row-0 granule; `dwave` is the
// wave's index among the waves that hold data.
template <int ROWS>
__device__ __forceinline__ int lane_tile_bytes(int dwave) {
    const int lane = threadIdx.x & (kWave - 1);
    return (dwave * (kWave * ROWS) + lane) * 16;
}

// ---------------------------------------------------------------------------
// Tile assignment.  The paper does not say how tiles get to workgroups (Sec. V-B);
// what the look-back needs is that the tile a workgroup waits for is owned by a
// workgroup that is running or will run without anybody's help.  Two ways:
//
//   by index    workgroup b takes tiles b, b + G, b + 2G, ... (G = grid size).  Safe as long as
//               every workgroup of the grid gets to run while the others wait, which holds
//               for G <= number of compute units: any compute unit can host one workgroup of
//               any kernel, and whatever else occupies the device finishes without our help.
//               The host uses it for exactly those grids, which covers every default shape
//               (one 1024-thread workgroup per compute unit; small inputs have few tiles).
//   by ticket   every tile, the first one included, comes from a counter in the call's
//               scratch.  Tickets go up and a workgroup handles its tiles in increasing
//               order, so the lowest unfinished tile always belongs to a running workgroup
//               that waits for nobody, whatever the grid size and however few workgroups are
//               resident.  Used for grids of more than one workgroup per compute unit (how
//               many of those the hardware really grants is not known: the runtime's
//               occupancy figure has been seen to say 8 where 7 ran), and on request.
//
// Tickets cost a little: all workgroups move in near lock-step, so their draws arrive in
// bursts on one address (12 ns each: the last of 256 waits 3 us), and the order of the tiles
// among neighbouring workgroups gets shuffled in every round, so a tile's predecessor is no
// longer always a little ahead of it.  Float32 sum, by index / by ticket, TB/s: 2^28 6.44 / 6.45,
// 2^26 6.14 / 6.04; arg-max struct 2^26 6.33 / 6.15.  Who draws matters more: a wave's vector memory
// operations return in order, and when the look-back wave drew, its first poll of every round
// waited behind the draw (float32 sum 2^28: 5.92).  So the first data wave draws, right before it
// requests the next tile: the ticket comes back ahead of 135 KiB of loads that the wave waits
// for anyway, and nobody ever waits for a ticket alone (except for the very first ones, at the
// start of the kernel).
//
// Control block: the first 4 KiB of the scratch, in 128-byte lines.  Line 0, word 0:
// tickets drawn; word 2 and lines 1 .. 16: the counters that tell which workgroup is
// the last one (of a launch by ticket; of a reduction, ks_reduce.hpp).  All are zero
// before a launch; the last workgroup puts them back to zero, so a library-owned
// scratch needs no clearing between calls.
// ---------------------------------------------------------------------------
constexpr size_t kControlBytes = 4096;
constexpr uint32_t kNoTile = 0xffffffffu;

// Who arrives last?  Workgroup b counts on the word of group b % kCountGroups (a 128-byte line
// each: lines 1 .. 16 of the control block); the one that completes its group counts the group
// on word 2 of line 0, and the one that completes the groups is the last workgroup of the grid.
// Atomics on ONE word are served one after the other, about 10 ns each: 512 workgroups counting on a
// single word cost 5 us.  Called by one thread per workgroup, when the workgroup is done.
constexpr uint32_t kCountGroups = 16;
constexpr uint32_t kLineWords = 32;
static_assert((1 + kCountGroups) * kLineWords * sizeof(uint32_t) <= kControlBytes, "the counters' lines must fit the control block");
__device__ __forceinline__ bool arrive_last(uint32_t *control) {
    const uint32_t g = blockIdx.x % kCountGroups;
    const uint32_t members = (gridDim.x - g + kCountGroups - 1) / kCountGroups;   // workgroups of this group
    if (__hip_atomic_fetch_add(&control[kLineWords * (1 + g)], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u != members)
        return false;
    const uint32_t groups = gridDim.x < kCountGroups ? gridDim.x : kCountGroups;
    return __hip_atomic_fetch_add(&control[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == groups;
}
// The last workgroup leaves the counters at zero for the next call.
__device__ __forceinline__ void reset_arrivals(uint32_t *control) {
    __hip_atomic_store(&control[2], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (uint32_t g = 0; g < kCountGroups; ++g)
        __hip_atomic_store(&control[kLineWords * (1 + g)], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}


// Issue a draw (one lane).
__device__ __forceinline__ uint32_t draw_ticket(uint32_t *control) {
    return __hip_atomic_fetch_add(&control[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by one lane of every workgroup of a launch by ticket, after its last draw has come back.
__device__ __forceinline__ void leave_grid(uint32_t *control) {
    if (arrive_last(control)) {
        __hip_atomic_store(&control[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        reset_arrivals(control);
    }
}

// Arguments of the look-back kernels that their loops pass around.
struct LookbackArgs {
    size_t n;
    uint32_t *control;       // control block (above)
    uint64_t *desc, *xdesc;
    uint32_t epoch, ntiles, spin_limit;
    uint32_t *abort_flag;    // abort word of the call's stream
    uint32_t call_seq;       // what a wave that gives up writes there; never zero
    uint32_t tickets;        // 0: tiles by index (grid <= tiles), 1: by ticket
    uint32_t seeded;         // 1: everything before element 0 is the value in line kSeedLine of the control block
};

// A seeded scan (out[i] = seed op in[0] op ... op in[i]: one piece of a longer sequence, scanned
// chunk by chunk or shard by shard).  Descriptors and look-back are those of the plain scan; the
// look-back wave puts the seed in front of the prefix it hands to its own workgroup's data waves.
// The launch stores the seed in the operator's chain type in line kSeedLine of the control block
// (seed_store_kernel) before the scan kernel starts.
constexpr uint32_t kSeedLine = 20;
template <class C, class COp>
__device__ __forceinline__ C seed_or_identity(const LookbackArgs &a) {
    if (!a.seeded) return COp::identity();
    typename WordsOf<C>::type w;
#pragma unroll
    for (int i = 0; i < WordsOf<C>::W; ++i) w.w[i] = a.control[kLineWords * kSeedLine + i];
    return from_words<C>(w);
}

// First tile of the calling workgroup (all threads call; kNoTile: nothing left, leave).
__device__ __forceinline__ uint32_t first_tile(const LookbackArgs &a, uint32_t *s_first) {
    if (!a.tickets) return blockIdx.x;
    if (threadIdx.x == 0) {
        const uint32_t t = draw_ticket(a.control);
        *s_first = t < a.ntiles ? t : kNoTile;
        if (t >= a.ntiles) leave_grid(a.control);
    }
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(*s_first);
}

// By ticket, round r of a workgroup handles tile t_r between two barriers A(r) and B(r).  The
// drawing wave (wave 1, lane 0) issues the draw of t_(r+1) in round r - 1, just before its loads
// of t_r, has the value when those loads are back at the top of round r, and writes it to
// next_tile before A(r); every wave reads it between A(r) and B(r).  The write for the round
// after comes after B(r).
struct TileQueue {
    uint32_t next_tile;
};
constexpr int kDrawingWave = 1;

// The tile after `tile`, read between the two barriers of a round (>= ntiles: none).
__device__ __forceinline__ uint32_t next_tile_of(const LookbackArgs &a, const TileQueue &q, uint32_t tile) {
    return a.tickets ? __builtin_amdgcn_readfirstlane(q.next_tile) : tile + gridDim.x;
}

// ---------------------------------------------------------------------------
// Single-pass scan.  The grid is persistent, about as many workgroups as fit the
// device, each taking tiles until none are left (tile assignment: above).  Every
// wait is bounded by spin_limit.
//
// IO = element type in memory, Op::acc = type of the registers, ChainOf<Op>::type = type of
// wave totals once they leave the wave, of aggregates and of descriptors.
// A workgroup has WAVES wave64s.  Wave 0 talks to the descriptors (publish,
// look-back).  In the 16-wave shape it does nothing else and waves 1..15 each
// own a run of 64*ROWS granules of the tile: vector memory instructions of a
// wave return in order, so a wave that also streams data sees every descriptor
// poll queue behind its own prefetch.  Measured on MI355X the dedicated wave
// is worth 7 % (float32 sum, n = 2^28: 5.70 -> 6.13 TB/s), more than the 1/16
// of the registers it leaves unused; in the 4- and 8-wave shapes it would idle
// 1/4 or 1/8 of the workgroup and wave 0 holds data like the others.
// With PREFETCH the next tile's granules are requested before the look-back
// wait and parked unconverted.
//
// The tile loop exists in three forms (template parameter FORM, below): one
// common loop for all waves in the 4- and 8-wave shapes; in the 16-wave shape
// loops of their own for the look-back wave and the data waves, which keeps the
// look-back's registers apart from the tile's (one register allocation serves
// the whole kernel: in a common loop the two add up, and a reload of a spilled
// register in the loop waits for every outstanding load, which cancels the
// prefetch); and the latter with the blocked arrangement of ks_tile.hpp.  Which
// one a type uses by default was measured (ks_launch.hpp).
// ---------------------------------------------------------------------------
constexpr bool dedicated_lookback_wave(int waves) { return waves >= 16; }
constexpr int data_waves(int waves) { return dedicated_lookback_wave(waves) ? waves - 1 : waves; }

// What the waves of a workgroup share: A = accumulation type, C = chain type.
template <class A, class C, int WAVES>
struct TileExchange {
    typename WordsOf<A>::type tot[WAVES];     // per wave: combination of its run
    typename WordsOf<C>::type carry[WAVES];   // per wave: combination of the runs before it (separate loops)
    typename WordsOf<C>::type prefix;         // exclusive prefix of the tile, from the look-back
    uint32_t ok;                              // 0: a wait was abandoned, everybody leaves
    TileQueue q;
    uint32_t first;
};

// Two pauses after the barrier that hands the wave totals over, in units of 64 cycles (s_sleep).
// The compute unit's L1 returns loads in order, so once the 135 KiB of the next tile are requested
// every poll of the look-back wave comes back behind them, 6-7 us later.  Therefore
//   - the data waves hold the request for the next tile back (kPrefetchHold), so that the aggregate
//     goes out and the first poll comes back before it, and
//   - the look-back wave waits a little before its first poll (kPollDelay < kPrefetchHold), so that
//     this poll, the one that is not caught behind the loads, already finds the aggregates its
//     neighbours publish at about the same moment.
// Measured on MI355X, separate loops, TB/s.  Hold alone, 0 / 12 / 24 / 32 / 48 / 96: uint64 sum
// 5.99 / 6.12 / 6.15 / 6.14 / 6.11 / 5.75, affine 5.14 / 5.82 / 5.84 / 5.82 / 5.81 / 5.53, arg-max struct
// 5.5 / 5.66 / 5.86 / 6.05 / 6.05 / 5.69, quaternions 5.3 / 5.60 / 5.90 / 5.91 / 5.89 / 5.70.  With the poll
// delay (delay / hold): uint64 0/32 6.17, 16/32 6.26, 24/40 6.28, 28/32 6.15; affine 0/32 5.82, 20/32
// 6.01, 24/40 5.99, 28/32 5.65; arg-max 0/32 6.05, 24/40 6.16, 28/44 6.17, 24/32 5.84: the hold has to
// exceed the delay by 12-16 for the poll to be issued first.  Releasing the request by a flag in LDS
// as soon as the aggregate is out, or when the look-back is done (bounded), measured 1-5 % below
// the fixed pauses.  Both apply only while the workgroup has a next tile to request.
// With the staggered start (below) accumulators of 16 bytes gain from longer pauses, 8-byte ones
// do not (delay / hold 24/40, 32/48, 40/56, 48/64 at 2 GiB of traffic: arg-max struct 6.25 / 6.30 / 6.32 /
// 6.33, quaternions 6.25 / 6.29 / 6.32 / 6.33, 2x2 matrices 6.35 / 6.38 / 6.40 / 6.40, affine 6.20 / 6.22 / 6.22 /
// 6.24, uint64 sum 6.43 / 6.43 / 6.43 / -; at 256 MiB of traffic 48/64 starts to lose).
constexpr int kPrefetchHold = 40;
constexpr int kPollDelay = 24;
constexpr int kPrefetchHoldWide = 56;   // accumulators of 16 bytes and more
constexpr int kPollDelayWide = 40;
template <class A>
constexpr int prefetch_hold() { return sizeof(A) >= 16 ? kPrefetchHoldWide : kPrefetchHold; }
template <class A>
constexpr int poll_delay() { return sizeof(A) >= 16 ? kPollDelayWide : kPollDelay; }
// Float32 sum, separate loops, delay / hold, TB/s at n = 2^28 / 2^26 / 2^24: 16/32 6.42 / 6.15 / 6.09, 24/40
// 6.42 / 6.13 / 6.07, 32/48 6.41 / 6.09 / 5.99, 40/56 6.39 / 6.04 / 5.90, 56/72 6.34 / 5.96 / 5.77.

// Output pointers that are not aligned to a 128-byte line (element-aligned views, paper
// Sec. IV-D).  The buffer accesses work at any alignment, but with tiles that start in the middle
// of a line every 1 KiB row of a wave straddles nine lines instead of covering eight, and the
// lines at the seams are written in two parts (float32 sum 2^28, both pointers moved by 4 bytes:
// 6.07 TB/s against 6.41).  So all tiles move down by `shift` elements: tile 0 keeps only the
// `lead` elements in front of the output's first line boundary and every other tile starts on a
// boundary (6.42 against 6.39 aligned in that run; with different offsets of input and output the
// loads stay off the lines, 6.29).  Host and kernel derive lead and shift from the output pointer alone.
template <class IO>
__host__ __device__ __forceinline__ uint32_t lead_elements(const IO *out) {
    return (uint32_t)((128u - (uint32_t)((uintptr_t)out & 127u)) & 127u) / (uint32_t)sizeof(IO);
}
template <class IO>
__host__ __device__ __forceinline__ size_t tile_shift(const IO *out, size_t tile_elems) {
    const uint32_t lead = lead_elements(out);
    return lead ? tile_elems - lead : 0;
}
// first element and element count of tile t under a shift
__device__ __forceinline__ size_t shifted_first(uint32_t t, size_t shift, size_t tile_elems) {
    return t ? (size_t)t * tile_elems - shift : 0;
}
__device__ __forceinline__ size_t shifted_elems(uint32_t t, size_t shift, size_t tile_elems) {
    return t ? tile_elems : tile_elems - shift;
}

// First thing wave 0 does once the tile's aggregate is known: successors only
// need the aggregate, so it goes out before anything else is queued.
template <class A, class Op>
__device__ __forceinline__ void publish_aggregate(const LookbackArgs &a, uint32_t tile, const A &aggregate) {
    if ((threadIdx.x & (kWave - 1)) != 0) return;
    if (tile == 0) {
        desc_publish<A>(a.desc, 0, a.epoch, kPrefix, aggregate);
        desc_publish<A>(a.xdesc, 0, a.epoch, kPrefix, Op::identity());   // nothing before tile 0
    } else {
        desc_publish<A>(a.desc, tile, a.epoch, kPartial, aggregate);
    }
}

// Find the tile's exclusive prefix, publish its inclusive prefix, and hand the
// exclusive prefix to the other waves through x.  Called by wave 0 only.
template <class A, class Op, class X>
__device__ __forceinline__ void resolve_prefix(const LookbackArgs &a, uint32_t tile, uint32_t m, const A &aggregate,
                                               X &x) {
    const int lane = threadIdx.x & (kWave - 1);
    Op op;
    A excl = Op::identity();
    bool ok = true;
    if (tile != 0) {
        ok = lookback<A, Op>(a.desc, a.xdesc, m, tile, a.epoch, a.spin_limit, a.abort_flag, a.call_seq, excl);
        if (ok && lane == 0) desc_publish<A>(a.desc, tile, a.epoch, kPrefix, op(excl, aggregate));
    }
    if (lane == 0) {
        // the descriptors are those of the plain scan; the seed goes in front of what this
        // workgroup's own waves apply
        if (a.seeded) excl = op(seed_or_identity<A, Op>(a), excl);
        x.prefix = to_words(excl);
        x.ok = ok ? 1u : 0u;
    }
}

// 16-wave shape, wave 0: no data.  Per tile: barrier (the data waves' totals are
// in LDS), scan them (lane l takes the total of data wave l: the inclusive scan
// gives the tile's aggregate, the exclusive one every data wave's carry), publish,
// look back, hand the prefix over, barrier.  The two loops below execute the
// same number of barriers per tile and leave together.
template <class Op, int WAVES, bool PREFETCH>
__device__ __forceinline__ void lookback_wave_loop(
    const LookbackArgs &a, TileExchange<typename Op::acc, typename ChainOf<Op>::type, WAVES> &x, uint32_t first) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    COp op;
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t m = (a.ntiles + kWindow - 1) / kWindow;   // row length of the transposed X array
    uint32_t tile = first;
    for (;;) {
        __syncthreads();
        const uint32_t next = next_tile_of(a, x.q, tile);
        C mine = COp::identity();
        if (lane < WAVES - 1) mine = convert<C>(from_words<A>(x.tot[lane + 1]));
        const C upto = wave_inclusive_scan(mine, op);
        const C aggregate = read_lane(upto, WAVES - 2);
        const C before = wave_shift_up(upto, COp::identity());
        if (lane < WAVES - 1) x.carry[lane + 1] = to_words(before);
        publish_aggregate<C, COp>(a, tile, aggregate);
        if (PREFETCH && next < a.ntiles) __builtin_amdgcn_s_sleep(poll_delay<A>());   // while the data waves hold
        resolve_prefix<C, COp>(a, tile, m, aggregate, x);
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(x.ok) == 0u) return;
        if (next >= a.ntiles) return;
        tile = next;
    }
}

// 16-wave shape, waves 1..15: the data.  Kept apart from the look-back code so
// that the registers of the tile and of the parked next tile do not have to
// coexist with the look-back's temporaries (one register allocation serves the
// whole kernel; in one common loop the two add up and wide element types spill).
template <class IO, class Op, int WAVES, int ROWS, bool INCLUSIVE, bool PREFETCH>
__device__ __forceinline__ void data_wave_loop(
    const IO *in, IO *out, const LookbackArgs &a,
    TileExchange<typename Op::acc, typename ChainOf<Op>::type, WAVES> &x, uint32_t first) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    typename ChainOf<Op>::op cop;
    using S = TileShape<IO, ROWS>;
    constexpr size_t TILE = (size_t)(WAVES - 1) * S::WAVE_ELEMS;
    // see pinned(): 4-byte elements measure 1 % faster without it (float32 sum 2^28 6.43 against 6.37 TB/s,
    // int32 sum 6.38 / 6.32), 8-byte ones 0.3-0.8 % slower (uint64 sum 6.42 / 6.43, 2^25 6.11 / 6.16)
    // (more than 9 rows of 4-byte elements need it to stay inside the 128 registers: 12 rows with the
    // next tile parked spill 70 registers without it and none with it)
    constexpr bool PIN = sizeof(IO) != 4 || ROWS > 9;
    Op op;
    const size_t shift = tile_shift(out, TILE);   // tiles start on 128-byte lines of the output
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;   // 1 .. WAVES-1
    const int lane_bytes = lane_tile_bytes<ROWS>(wave - 1);
    const bool drawing = a.tickets && wave == kDrawingWave && lane == 0;
    uint32_t drawn = 0;   // drawing lane: the ticket of the tile after the one in `cur`
    if (drawing) drawn = draw_ticket(a.control);
    ThreadItems<A, ROWS, S::G> cur;
    load_items<IO, ROWS, Op, PIN>(tile_window<IO>(in, a.n, shifted_first(first, shift, TILE), shifted_elems(first, shift, TILE)), lane_bytes,
                             first + 1 == a.ntiles || (first == 0 && shift != 0), cur);
    uint32_t loop_tile = first;
    for (;;) {
        // The tile index is the same in every lane; saying so keeps it, and the buffer resources
        // derived from it, in scalar registers.
        const uint32_t tile = __builtin_amdgcn_readfirstlane(loop_tile);
        if (drawing) x.q.next_tile = drawn;
        // Commutative operators: the run's total first, by the shortest route, and the scan itself
        // after the barrier (see reduce_wave_run_any_order).  From the scan on `cur` holds the scan
        // of the wave's run alone.
        if constexpr (Op::commutative) {
            const A wave_total = reduce_wave_run_any_order<A, ROWS, S::G, Op>(cur, op);
            if (lane == 0) x.tot[wave] = to_words(wave_total);
        } else {
            const A wave_total = scan_wave_run_in_place<INCLUSIVE, A, ROWS, S::G, Op>(cur, op);
            if (lane == 0) x.tot[wave] = to_words(wave_total);
        }
        __syncthreads();
        // The next tile is requested only now, after the totals are out: requested before the scan
        // (the registers would be free) it measured 5-12 % slower, the descriptor traffic of the
        // look-back wave then queues behind 135 KiB of loads in this compute unit's memory pipeline.
        const uint32_t next = next_tile_of(a, x.q, tile);
        if (drawing && next < a.ntiles) drawn = draw_ticket(a.control);   // no draw once one has failed
        RawItems<ROWS> nxt;
        TileWindow wnext;
        if (PREFETCH && next < a.ntiles) {
            __builtin_amdgcn_s_sleep(prefetch_hold<A>());
            wnext = tile_window<IO>(in, a.n, (size_t)next * TILE - shift, TILE);
            load_raw<ROWS, PIN>(wnext, lane_bytes, nxt);
        }
        if constexpr (Op::commutative) (void)scan_wave_run_in_place<INCLUSIVE, A, ROWS, S::G, Op>(cur, op);
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(x.ok) == 0u) break;
        const A prefix = convert<A>(cop(from_words<C>(x.prefix), from_words<C>(x.carry[wave])));
        apply_prefix_and_store<IO, ROWS, A, Op, PIN>(tile_window<IO>(out, a.n, shifted_first(tile, shift, TILE), shifted_elems(tile, shift, TILE)), lane_bytes, cur,
                                                prefix, op);
        if (next >= a.ntiles) break;
        loop_tile = next;
        if (PREFETCH) {
            unpack_items<IO, ROWS, Op, PIN>(nxt, lane_bytes, wnext.valid_bytes, next + 1 == a.ntiles, cur);
        } else {
            load_items<IO, ROWS, Op, PIN>(tile_window<IO>(in, a.n, (size_t)next * TILE - shift, TILE), lane_bytes,
                                     next + 1 == a.ntiles, cur);
        }
    }
    if (drawing) leave_grid(a.control);   // `drawn` has been used: the last draw is back
}

// The data waves of the 16-wave shape in the blocked arrangement (ks_tile.hpp):
// same protocol and barriers as data_wave_loop, but every wave passes its
// granules through its LDS region `stage + (wave - 1) * Stage<ROWS>::SLOTS` on
// the way in and on the way out, and scans ROWS consecutive granules per lane.
template <class IO, class Op, int WAVES, int ROWS, bool INCLUSIVE, bool PREFETCH>
__device__ __forceinline__ void blocked_data_wave_loop(
    const IO *in, IO *out, const LookbackArgs &a,
    TileExchange<typename Op::acc, typename ChainOf<Op>::type, WAVES> &x, u32x4 *stage, uint32_t first) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    typename ChainOf<Op>::op cop;
    using S = BlockedShape<IO, ROWS>;
    constexpr size_t TILE = (size_t)(WAVES - 1) * S::WAVE_ELEMS;
    Op op;
    const size_t shift = tile_shift(out, TILE);   // see data_wave_loop
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;   // 1 .. WAVES-1
    const int lane_bytes = lane_tile_bytes<ROWS>(wave - 1);   // striped view: global loads and stores
    const int run_bytes = (wave - 1) * (kWave * ROWS * 16);   // start of the wave's run inside the tile
    u32x4 *region = stage + (wave - 1) * Stage<ROWS>::SLOTS;
    // The next tile is requested after the totals are out and the pause of kPrefetchHold, as in
    // data_wave_loop.  (Requested before the scan, which looked best for 16-byte elements while
    // nothing kept the request from overtaking the look-back's polls, it measures 8-11 % below
    // the held request: arg-max struct 5.59 against 6.05 TB/s.)
    const bool drawing = a.tickets && wave == kDrawingWave && lane == 0;   // see data_wave_loop
    uint32_t drawn = 0;
    if (drawing) drawn = draw_ticket(a.control);
    RawItems<ROWS> raw;
    uint32_t valid_bytes;
    {
        const TileWindow w = tile_window<IO>(in, a.n, shifted_first(first, shift, TILE), shifted_elems(first, shift, TILE));
        load_raw<ROWS, true>(w, lane_bytes, raw);
        valid_bytes = w.valid_bytes;
    }
    uint32_t loop_tile = first;
    for (;;) {
        const uint32_t tile = __builtin_amdgcn_readfirstlane(loop_tile);   // see data_wave_loop
        if (drawing) x.q.next_tile = drawn;
        LaneItems<A, S::E> cur;
        A lane_before;
        striped_to_blocked<ROWS>(region, raw);
        unpack_blocked<IO, ROWS, Op>(raw, run_bytes, valid_bytes, tile + 1 == a.ntiles || (tile == 0 && shift != 0), cur);
        const A wave_total = scan_blocked_run<A, S::E, Op>(cur, lane_before, op);
        if (lane == 0) x.tot[wave] = to_words(wave_total);
        __syncthreads();
        const uint32_t next = next_tile_of(a, x.q, tile);
        if (drawing && next < a.ntiles) drawn = draw_ticket(a.control);
        if (PREFETCH && next < a.ntiles) {
            __builtin_amdgcn_s_sleep(prefetch_hold<A>());
            const TileWindow w = tile_window<IO>(in, a.n, (size_t)next * TILE - shift, TILE);
            load_raw<ROWS, true>(w, lane_bytes, raw);
            valid_bytes = w.valid_bytes;
        }
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(x.ok) == 0u) break;
        const A before = op(convert<A>(cop(from_words<C>(x.prefix), from_words<C>(x.carry[wave]))), lane_before);
        RawItems<ROWS> result;
        apply_blocked<INCLUSIVE, IO, ROWS, A, Op>(cur, before, op, result);
        blocked_to_striped<ROWS>(region, result);
        store_raw<ROWS, true>(tile_window<IO>(out, a.n, shifted_first(tile, shift, TILE), shifted_elems(tile, shift, TILE)), lane_bytes, result);
        if (next >= a.ntiles) break;
        loop_tile = next;
        if (!PREFETCH) {
            const TileWindow w = tile_window<IO>(in, a.n, (size_t)next * TILE - shift, TILE);
            load_raw<ROWS, true>(w, lane_bytes, raw);
            valid_bytes = w.valid_bytes;
        }
    }
    if (drawing) leave_grid(a.control);
}

// What the waves share in the common loop.
template <class A, class C, int WAVES>
struct CommonExchange {
    typename WordsOf<A>::type tot[WAVES];
    typename WordsOf<C>::type prefix;
    uint32_t ok;
    TileQueue q;
    uint32_t first;
};

// One loop for all waves (the 4- and 8-wave shapes): every wave holds data and
// wave 0 looks back as well; wave 1 draws the tickets.
template <class IO, class Op, int WAVES, int ROWS, bool INCLUSIVE, bool PREFETCH>
__device__ __forceinline__ void common_wave_loop(
    const IO *in, IO *out, const LookbackArgs &a,
    CommonExchange<typename Op::acc, typename ChainOf<Op>::type, WAVES> &x, uint32_t first) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    using S = TileShape<IO, ROWS>;
    using Items = ThreadItems<A, ROWS, S::G>;
    constexpr size_t TILE = (size_t)WAVES * S::WAVE_ELEMS;
    Op op;
    COp cop;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const bool lookback_wave = wave == 0;
    const int lane_bytes = lane_tile_bytes<ROWS>(wave);
    const uint32_t m = (a.ntiles + kWindow - 1) / kWindow;   // row length of the transposed X array

    uint32_t tile = first;
    const bool drawing = a.tickets && wave == kDrawingWave && lane == 0;   // see data_wave_loop
    uint32_t drawn = 0;
    if (drawing) drawn = draw_ticket(a.control);
    Items cur;
    load_items<IO, ROWS, Op, false>(tile_window<IO>(in, a.n, (size_t)tile * TILE, TILE), lane_bytes, tile + 1 == a.ntiles, cur);
    for (;;) {
        if (drawing) x.q.next_tile = drawn;
        WaveScan<A, ROWS> ws = scan_wave_run<A, ROWS, S::G, Op>(cur, op);
        C aggregate;
        const C wave_carry = exchange_wave_totals<Op, WAVES>(x.tot, ws.wave_total, aggregate);

        // publish as early as possible: successors only need the aggregate
        if (lookback_wave && lane == 0) {
            desc_publish<C>(a.desc, tile, a.epoch, tile == 0 ? kPrefix : kPartial, aggregate);
            if (tile == 0) desc_publish<C>(a.xdesc, 0, a.epoch, kPrefix, COp::identity());   // nothing before tile 0
        }
        const uint32_t next = next_tile_of(a, x.q, tile);
        const bool more = next < a.ntiles;
        if (drawing && more) drawn = draw_ticket(a.control);   // no draw once one has failed
        RawItems<ROWS> nxt;
        TileWindow wnext;
        if (PREFETCH && more) {
            wnext = tile_window<IO>(in, a.n, (size_t)next * TILE, TILE);
            load_raw<ROWS, false>(wnext, lane_bytes, nxt);
        }
        if (lookback_wave) {
            C excl = COp::identity();
            bool ok = true;
            if (tile != 0) {
                ok = lookback<C, COp>(a.desc, a.xdesc, m, tile, a.epoch, a.spin_limit, a.abort_flag, a.call_seq, excl);
                if (ok && lane == 0) desc_publish<C>(a.desc, tile, a.epoch, kPrefix, cop(excl, aggregate));
            }
            if (lane == 0) {
                if (a.seeded) excl = cop(seed_or_identity<C, COp>(a), excl);   // see resolve_prefix
                x.prefix = to_words(excl);
                x.ok = ok ? 1u : 0u;
            }
        }
        __syncthreads();
        if (x.ok == 0u) break;   // a wait was abandoned: the host reports KS_ERR_TIMEOUT

        const A prefix = convert<A>(cop(from_words<C>(x.prefix), wave_carry));
        finish_wave_run<INCLUSIVE, A, ROWS, S::G, Op>(cur, ws, op);
        apply_prefix_and_store<IO, ROWS, A, Op, false>(tile_window<IO>(out, a.n, (size_t)tile * TILE, TILE), lane_bytes, cur,
                                                       prefix, op);
        if (!more) break;
        tile = next;
        if (PREFETCH)
            unpack_items<IO, ROWS, Op, false>(nxt, lane_bytes, wnext.valid_bytes, tile + 1 == a.ntiles, cur);
        else
            load_items<IO, ROWS, Op, false>(tile_window<IO>(in, a.n, (size_t)tile * TILE, TILE), lane_bytes, tile + 1 == a.ntiles, cur);
    }
    if (drawing) leave_grid(a.control);
}

// Staggered start (16-wave shape, one workgroup per compute unit).  Left alone, all workgroups
// request their first tile in the same instant and then move in lock-step rounds, so that the whole
// chip reads at one time and writes at another.  Spreading the starts over about a third of a round
// (workgroup b waits b / grid of kStartStagger x 64 cycles) lets reads and writes of different compute
// units overlap and every tile find its predecessors' descriptors already there.  Measured, TB/s,
// stagger 0 / 75 / 150 / 300: float32 sum 2^28 6.29 / 6.40 / 6.45 / 6.34, 2^26 5.78 / 6.05 / 6.12 / -,
// uint64 sum 2^27 6.33 / 6.39 / 6.43 / 6.33, 2^25 5.83 / 6.11 / 6.15 / -, arg-max struct 2^26 6.14 / - / 6.25 /
// 6.18, 2^24 5.60 / 5.84 / 5.91 / -, affine 2^26 5.97 / - / 6.18 (100) / 6.05.  With fewer than about
// three rounds per workgroup the wait costs more than it gives (float32 2^24, 1.9 rounds: 5.95 / 5.68 /
// 5.36), so it applies from kStaggerFromRounds rounds on.
constexpr uint32_t kStartStagger = 150;
constexpr uint32_t kStaggerFromRounds = 3;

__device__ __forceinline__ void stagger_start(uint32_t ntiles, uint32_t first) {
    if (ntiles < kStaggerFromRounds * gridDim.x) return;
    const uint32_t pauses = (first % gridDim.x) * kStartStagger / gridDim.x;   // first: the workgroup's first tile
    for (uint32_t i = 0; i < pauses; ++i) __builtin_amdgcn_s_sleep(1);
}

// FORM: which loop the kernel runs (see above).
constexpr int kFormCommon = 0;     // one loop for all waves (4- and 8-wave shapes)
constexpr int kFormSeparate = 1;   // 16 waves: look-back wave and data waves in loops of their own, striped items
constexpr int kFormBlocked = 2;    // the same with the blocked arrangement (LDS exchange)
constexpr int kFormCount = 3;
// whether the kernel of this shape moves its tiles to the output's line boundaries
constexpr bool aligns_output(int waves) { return dedicated_lookback_wave(waves); }

template <class IO, class Op, int WAVES, int ROWS, bool INCLUSIVE, bool PREFETCH, int FORM>
__global__ __launch_bounds__(WAVES *kWave) void scan_lookback_kernel(const IO *in, IO *out, LookbackArgs a) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    static_assert(dedicated_lookback_wave(WAVES) == (FORM != kFormCommon), "16 waves run separate loops, 4 and 8 the common one");
    if constexpr (dedicated_lookback_wave(WAVES)) {
        __shared__ TileExchange<A, C, WAVES> x;
        const uint32_t first = first_tile(a, &x.first);
        if (first == kNoTile) return;
        stagger_start(a.ntiles, first);
        if constexpr (FORM == kFormBlocked) {
            __shared__ u32x4 stage[(WAVES - 1) * Stage<ROWS>::SLOTS];
            if (threadIdx.x < kWave)
                lookback_wave_loop<Op, WAVES, PREFETCH>(a, x, first);
            else
                blocked_data_wave_loop<IO, Op, WAVES, ROWS, INCLUSIVE, PREFETCH>(in, out, a, x, stage, first);
        } else {
            if (threadIdx.x < kWave)
                lookback_wave_loop<Op, WAVES, PREFETCH>(a, x, first);
            else
                data_wave_loop<IO, Op, WAVES, ROWS, INCLUSIVE, PREFETCH>(in, out, a, x, first);
        }
    } else {
        __shared__ CommonExchange<A, C, WAVES> x;
        const uint32_t first = first_tile(a, &x.first);
        if (first == kNoTile) return;
        common_wave_loop<IO, Op, WAVES, ROWS, INCLUSIVE, PREFETCH>(in, out, a, x, first);
    }
}

// ---------------------------------------------------------------------------
// Reduce-then-scan (no waiting between workgroups; one workgroup per tile).
// Aggregates and seeds are arrays of the operator's chain type.
// ---------------------------------------------------------------------------
// BLOCKED: the blocked arrangement of ks_tile.hpp (every wave exchanges its granules through a
// region of LDS of its own), which is what serves element sizes other than 4, 8 and 16 bytes;
// otherwise the striped arrangement.
template <class IO, int ROWS, bool BLOCKED>
constexpr size_t rts_tile_elems() {
    if constexpr (BLOCKED) return (size_t)kWaves * BlockedShape<IO, ROWS>::WAVE_ELEMS;
    else return (size_t)kWaves * TileShape<IO, ROWS>::WAVE_ELEMS;
}

template <class IO, class Op, int ROWS, bool BLOCKED>
__global__ __launch_bounds__(kBlock) void tile_reduce_kernel(const IO *__restrict__ in, size_t n,
                                                             typename ChainOf<Op>::type *__restrict__ aggregates) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    constexpr size_t TILE = rts_tile_elems<IO, ROWS, BLOCKED>();
    __shared__ typename WordsOf<A>::type s_tot[kWaves];
    Op op;
    const size_t tile = blockIdx.x;
    const int wave = threadIdx.x >> 6;
    const int lane_bytes = lane_tile_bytes<ROWS>(wave);
    const TileWindow w = tile_window<IO>(in, n, tile * TILE, TILE);
    const bool partial = (tile + 1) * TILE > n;
    A wave_total;
    if constexpr (BLOCKED) {
        __shared__ u32x4 stage[kWaves * Stage<ROWS>::SLOTS];
        RawItems<ROWS> raw;
        load_raw<ROWS, false>(w, lane_bytes, raw);
        striped_to_blocked<ROWS>(stage + wave * Stage<ROWS>::SLOTS, raw);
        LaneItems<A, BlockedShape<IO, ROWS>::E> cur;
        unpack_blocked<IO, ROWS, Op>(raw, wave * (kWave * ROWS * 16), w.valid_bytes, partial, cur);
        A lane_before;
        wave_total = scan_blocked_run<A, BlockedShape<IO, ROWS>::E, Op>(cur, lane_before, op);
    } else {
        using S = TileShape<IO, ROWS>;
        ThreadItems<A, ROWS, S::G> cur;
        load_items<IO, ROWS, Op, false>(w, lane_bytes, partial, cur);
        wave_total = scan_wave_run<A, ROWS, S::G, Op>(cur, op).wave_total;
    }
    C aggregate;
    (void)exchange_wave_totals<Op, kWaves>(s_tot, wave_total, aggregate);
    if (threadIdx.x == 0) aggregates[tile] = aggregate;
}

// seeds == nullptr: every tile starts from the identity (used when one tile
// covers the whole input).  Otherwise seeds[tile] = combination of all earlier tiles.
template <class IO, class Op, int ROWS, bool INCLUSIVE, bool BLOCKED>
__global__ __launch_bounds__(kBlock) void tile_scan_kernel(const IO *in, IO *out, size_t n,
                                                           const typename ChainOf<Op>::type *__restrict__ seeds) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    COp cop;
    constexpr size_t TILE = rts_tile_elems<IO, ROWS, BLOCKED>();
    __shared__ typename WordsOf<A>::type s_tot[kWaves];
    Op op;
    const size_t tile = blockIdx.x;
    const int wave = threadIdx.x >> 6;
    const int lane_bytes = lane_tile_bytes<ROWS>(wave);
    const TileWindow w = tile_window<IO>(in, n, tile * TILE, TILE);
    const TileWindow wo = tile_window<IO>(out, n, tile * TILE, TILE);
    const bool partial = (tile + 1) * TILE > n;
    const C seed = seeds ? seeds[tile] : COp::identity();
    if constexpr (BLOCKED) {
        __shared__ u32x4 stage[kWaves * Stage<ROWS>::SLOTS];
        u32x4 *region = stage + wave * Stage<ROWS>::SLOTS;
        RawItems<ROWS> raw;
        load_raw<ROWS, false>(w, lane_bytes, raw);
        striped_to_blocked<ROWS>(region, raw);
        LaneItems<A, BlockedShape<IO, ROWS>::E> cur;
        unpack_blocked<IO, ROWS, Op>(raw, wave * (kWave * ROWS * 16), w.valid_bytes, partial, cur);
        A lane_before;
        const A wave_total = scan_blocked_run<A, BlockedShape<IO, ROWS>::E, Op>(cur, lane_before, op);
        C aggregate;
        const C wave_carry = exchange_wave_totals<Op, kWaves>(s_tot, wave_total, aggregate);
        const A before = op(convert<A>(cop(seed, wave_carry)), lane_before);
        RawItems<ROWS> result;
        apply_blocked<INCLUSIVE, IO, ROWS, A, Op>(cur, before, op, result);
        blocked_to_striped<ROWS>(region, result);
        store_raw<ROWS, false>(wo, lane_bytes, result);
    } else {
        using S = TileShape<IO, ROWS>;
        ThreadItems<A, ROWS, S::G> cur;
        load_items<IO, ROWS, Op, false>(w, lane_bytes, partial, cur);
        const WaveScan<A, ROWS> ws = scan_wave_run<A, ROWS, S::G, Op>(cur, op);
        C aggregate;
        const C wave_carry = exchange_wave_totals<Op, kWaves>(s_tot, ws.wave_total, aggregate);
        finish_wave_run<INCLUSIVE, A, ROWS, S::G, Op>(cur, ws, op);
        apply_prefix_and_store<IO, ROWS, A, Op, false>(wo, lane_bytes, cur, convert<A>(cop(seed, wave_carry)), op);
    }
}

// Single-pass scan of a strided view (element i at base[i * stride], paper Sec. IV-C): the
// look-back protocol of scan_lookback_kernel (Sec. V-B) with one-element accesses and one-element
// granules (a tile is 4 waves x ROWS rows x 64 elements).  Four waves, all holding data, no
// prefetch: a strided access pattern is bound by the sectors it touches, and many small workgroups
// per compute unit keep more of them in flight than one large one.
template <class IO, class Op, int WAVES, int ROWS, bool INCLUSIVE>
__global__ __launch_bounds__(WAVES *kWave) void scan_lookback_strided_kernel(const IO *in, size_t in_stride, IO *out,
                                                                       size_t out_stride, LookbackArgs a) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    constexpr size_t WAVE_ELEMS = (size_t)kWave * ROWS;   // one-element granules
    constexpr size_t TILE = (size_t)WAVES * WAVE_ELEMS;
    __shared__ CommonExchange<A, C, WAVES> x;
    Op op;
    COp cop;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const uint32_t m = (a.ntiles + kWindow - 1) / kWindow;   // row length of the transposed X array
    uint32_t tile = first_tile(a, &x.first);
    if (tile == kNoTile) return;
    for (;;) {
        const size_t run_first = (size_t)tile * TILE + (size_t)wave * WAVE_ELEMS;
        ThreadItems<A, ROWS, 1> cur;
        load_items_strided<IO, ROWS, Op>(in, in_stride, a.n, run_first, cur);
        const WaveScan<A, ROWS> ws = scan_wave_run<A, ROWS, 1, Op>(cur, op);
        C aggregate;
        const C wave_carry = exchange_wave_totals<Op, WAVES>(x.tot, ws.wave_total, aggregate);
        // no prefetch here: the next tile is only needed after the closing barrier; wave 1 draws it
        // now and has it long before wave 0 is back from the look-back
        if (a.tickets && wave == kDrawingWave && lane == 0) x.q.next_tile = draw_ticket(a.control);
        if (wave == 0) {
            if (lane == 0) {
                desc_publish<C>(a.desc, tile, a.epoch, tile == 0 ? kPrefix : kPartial, aggregate);
                if (tile == 0) desc_publish<C>(a.xdesc, 0, a.epoch, kPrefix, COp::identity());   // nothing before tile 0
            }
            C excl = COp::identity();
            bool ok = true;
            if (tile != 0) {
                ok = lookback<C, COp>(a.desc, a.xdesc, m, tile, a.epoch, a.spin_limit, a.abort_flag, a.call_seq, excl);
                if (ok && lane == 0) desc_publish<C>(a.desc, tile, a.epoch, kPrefix, cop(excl, aggregate));
            }
            if (lane == 0) {
                x.prefix = to_words(excl);
                x.ok = ok ? 1u : 0u;
            }
        }
        __syncthreads();
        if (x.ok == 0u) break;   // a wait was abandoned: the host reports KS_ERR_TIMEOUT
        const A prefix = convert<A>(cop(from_words<C>(x.prefix), wave_carry));
        finish_wave_run<INCLUSIVE, A, ROWS, 1, Op>(cur, ws, op);
        apply_prefix_and_store_strided<IO, ROWS, A, Op>(out, out_stride, a.n, run_first, cur, prefix, op);
        // next_tile is written between the two barriers of a round and read after the second one;
        // the next write comes after the first barrier of the next round (inside exchange_wave_totals)
        tile = next_tile_of(a, x.q, tile);
        if (tile >= a.ntiles) break;
    }
    if (a.tickets && threadIdx.x == kDrawingWave * kWave) leave_grid(a.control);
}

// The seed of a seeded scan, one element of the caller's in the element type, goes into the control
// block in the chain type.  A map that changes the type promotes it (16-bit floats); any other map is
// not applied: the seed is a value already accumulated, not an input element.
template <class IO, class Op>
__global__ void seed_store_kernel(const IO *seed, uint32_t *control) {
    using A = typename Op::acc;
    using C = typename ChainOf<Op>::type;
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    A v;
    if constexpr (ResultOf<Op, IO>::from_map) v = convert<A>(typename MapOf<Op>::type()(seed[0]));
    else v = convert<A>(seed[0]);
    const typename WordsOf<C>::type w = to_words(convert<C>(v));
    for (int i = 0; i < WordsOf<C>::W; ++i) control[kLineWords * kSeedLine + i] = w.w[i];
}

template <int UNUSED = 0>
__global__ void fill_zero_kernel(uint64_t *p, size_t words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < words; i += stride) p[i] = 0ull;
}

// Vectorised copy, one 16-byte granule per lane and ROWS granules per thread in
// the same wave-run arrangement as the scan (paper Sec. IV-C, copy kernel).
template <int ROWS>
__global__ __launch_bounds__(kBlock) void copy_kernel(const u32x4 *__restrict__ in, u32x4 *__restrict__ out,
                                                      size_t granules) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const size_t first = ((size_t)blockIdx.x * kWaves + wave) * (size_t)(kWave * ROWS) + lane;
    u32x4 v[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const size_t i = first + (size_t)j * kWave;
        if (i < granules) v[j] = __builtin_nontemporal_load(in + i);
    }
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const size_t i = first + (size_t)j * kWave;
        if (i < granules) __builtin_nontemporal_store(v[j], out + i);
    }
}

}  // namespace ks
