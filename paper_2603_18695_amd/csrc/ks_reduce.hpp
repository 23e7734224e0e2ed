// mapreduce(f, op, src) in one launch (paper Sec. II-C: op(f(src[1]), ..., f(src[n])); Sec. V-A:
// fixed grid, partial results in registers, wave-level reduction by shuffles, cross-wave step
// through shared memory, one partial per workgroup in global memory, one workgroup finishes).
//
// What is kept from the paper's design: a fixed grid whatever n, register accumulation, DPP
// wave reduction, LDS across waves, a single launch.  What differs, and why:
//   - The unit of work is a run (64 lanes x ROWS 16-byte granules: the same coalesced buffer
//     loads and register arrangement as the scan).  For commutative operators a wave strides
//     over the runs as the paper's threads stride over the elements, every lane folds its own
//     items and one DPP reduction comes at the very end.  For the others a wave folds a
//     CONTIGUOUS range of runs in order: each run goes through the wave's LDS region into the
//     blocked arrangement (a lane holds ROWS consecutive granules), every lane folds its own
//     elements in sequence and ONE ordered DPP reduction combines the lanes; since the partials
//     are combined in workgroup order the result is the left fold: operators that do not commute
//     are served too, which the paper's strided accumulation cannot do.  Element sizes that do
//     not divide a granule (12, 24, 32 bytes) take this path whatever the operator.
//   - No designated workgroup that spins on flags: the workgroup that arrives LAST folds the
//     partials, so nobody waits for a workgroup that has not run.  Who is last is counted in two
//     levels, 16 groups of workgroups and the groups: atomics on one address are served one
//     after the other, about 10 ns each, and 512 workgroups counting on one word cost 5 us.
//   - Partials travel as tagged 64-bit words (ks_kernels.hpp, descriptors): value and flag in
//     one relaxed atomic instead of a release store and acquire loads; the finishing wave
//     polls the tags (bounded) rather than relying on the order of the counter and the data.
//   - Accumulation above one run is in the operator's chain type (double for float32 sums).
#pragma once

#include "ks_kernels.hpp"

namespace ks {

struct ReduceArgs {
    size_t n;
    size_t total_runs;
    uint32_t *control;     // control block of the scratch: the counters of arrive_last
    uint64_t *partials;    // gridDim.x entries of tagged words
    uint32_t epoch, spin_limit;
    uint32_t *abort_flag;
    uint32_t call_seq;
    uint32_t runs_per_wave;   // ordered (non-commutative) operators: contiguous runs per wave
    uint32_t head_skip;       // elements narrower than a dword: `in` was moved down to a dword boundary,
                              // and this many leading bytes of run 0 are not part of the input
};

constexpr int kFinishWindows = 4;   // windows of 64 partials a finishing wave has in flight at once

// ordered_reduction<IO, Op>(): contiguous ranges and the blocked arrangement instead of strided runs
template <class IO, class Op>
constexpr bool ordered_reduction() { return !Op::commutative || 16 % sizeof(IO) != 0; }

// One run folded by its wave, any order allowed: the lane's own items, nothing across lanes.
template <class IO, class Op, int ROWS>
__device__ __forceinline__ typename Op::acc fold_run_lane_private(const RawItems<ROWS> &raw, int lane_bytes,
                                                                  uint32_t valid_bytes, bool partial, uint32_t head_skip) {
    using A = typename Op::acc;
    using S = TileShape<IO, ROWS>;
    Op op;
    ThreadItems<A, ROWS, S::G> it;
    unpack_items<IO, ROWS, Op, false>(raw, lane_bytes, valid_bytes, partial, it);
    if constexpr (sizeof(IO) < 4) {
        if (head_skip != 0) {   // the bytes in front of the caller's first element
#pragma unroll
            for (int k = 0; k < S::G; ++k)
                if (lane_bytes + k * (int)sizeof(IO) < (int)head_skip) it.x[0][k] = Op::identity();
        }
    }
    A mine = it.x[0][0];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
#pragma unroll
        for (int k = 0; k < S::G; ++k)
            if (j != 0 || k != 0) mine = op(mine, it.x[j][k]);
    }
    return mine;
}

// One run folded in order: through `region` (the wave's own LDS) into the blocked arrangement,
// the lane's consecutive elements in sequence, then the lanes in order.  The same value in every lane.
template <class IO, class Op, int ROWS>
__device__ __forceinline__ typename Op::acc fold_run_in_order(u32x4 *region, RawItems<ROWS> raw, uint32_t valid_bytes,
                                                              bool partial) {
    using A = typename Op::acc;
    constexpr int E = BlockedShape<IO, ROWS>::E;
    Op op;
    striped_to_blocked<ROWS>(region, raw);
    LaneItems<A, E> it;
    unpack_blocked<IO, ROWS, Op>(raw, 0, valid_bytes, partial, it);
    A mine = it.y[0];
#pragma unroll
    for (int k = 1; k < E; ++k) mine = op(mine, it.y[k]);
    return read_lane(wave_inclusive_scan(mine, op), kWave - 1);
}

template <class IO, class Op, int ROWS>
__global__ __launch_bounds__(kBlock) void mapreduce_kernel(const IO *in, typename ResultOf<Op, IO>::type *out,
                                                           ReduceArgs a) {
    using A = typename Op::acc;
    using R = typename ResultOf<Op, IO>::type;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    constexpr bool ORDERED = ordered_reduction<IO, Op>();
    constexpr size_t RUN = (size_t)kWave * ROWS * 16 / sizeof(IO);   // elements of one run
    __shared__ typename WordsOf<C>::type s_tot[kWaves];
    __shared__ uint32_t s_last;
    __shared__ u32x4 s_stage[ORDERED ? kWaves * Stage<ROWS>::SLOTS : 1];
    COp cop;
    const int lane = threadIdx.x & (kWave - 1);
    // uniform for the compiler too: the runs' buffer descriptors then stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane_bytes = lane * 16;
    const size_t gw = (size_t)blockIdx.x * kWaves + wave;
    // any order: runs gw, gw + W, gw + 2W, ... (W = waves of the grid); ordered: a contiguous range
    const size_t step = ORDERED ? 1 : (size_t)gridDim.x * kWaves;
    size_t run = ORDERED ? gw * a.runs_per_wave : gw;
    size_t end = ORDERED ? run + a.runs_per_wave : a.total_runs;
    if (end > a.total_runs) end = a.total_runs;

    // Any order: acc is the lane's own running value.  Ordered: the wave's, the same in every lane.
    C acc = COp::identity();
    RawItems<ROWS> raw;
    TileWindow w;
    if (run < end) {
        w = tile_window<IO>(in, a.n, run * RUN, RUN);
        load_raw<ROWS, false>(w, lane_bytes, raw);
    }
    for (; run < end; run += step) {
        RawItems<ROWS> nxt;
        TileWindow wn;
        if (run + step < end) {   // the next run is on its way while this one is folded
            wn = tile_window<IO>(in, a.n, (run + step) * RUN, RUN);
            load_raw<ROWS, false>(wn, lane_bytes, nxt);
        }
        const bool partial = (run + 1) * RUN > a.n;
        if constexpr (ORDERED) {
            acc = cop(acc, convert<C>(fold_run_in_order<IO, Op, ROWS>(s_stage + wave * Stage<ROWS>::SLOTS, raw,
                                                                      w.valid_bytes, partial)));
        } else {
            acc = cop(acc, convert<C>(fold_run_lane_private<IO, Op, ROWS>(raw, lane_bytes, w.valid_bytes, partial,
                                                                          run == 0 ? a.head_skip : 0u)));
        }
        if (run + step < end) {
            raw = nxt;
            w = wn;
        }
    }
    if constexpr (!ORDERED) acc = read_lane(wave_inclusive_scan(acc, cop), kWave - 1);
    if (lane == 0) s_tot[wave] = to_words(acc);
    __syncthreads();
    if (threadIdx.x == 0) {
        C partial = from_words<C>(s_tot[0]);
#pragma unroll
        for (int k = 1; k < kWaves; ++k) partial = cop(partial, from_words<C>(s_tot[k]));
        desc_publish<C>(a.partials, blockIdx.x, a.epoch, kPartial, partial);
        s_last = arrive_last(a.control) ? 1u : 0u;
    }
    __syncthreads();
    if (s_last == 0u) return;

    // The last workgroup to arrive folds the partials in workgroup order: each of its waves takes a
    // contiguous quarter, kFinishWindows windows of 64 at a time (all their loads in flight together:
    // one memory round trip for 256 partials), thread 0 combines the four.
    const uint32_t quarter = ((gridDim.x + kWaves - 1) / kWaves + kWave - 1) / kWave * kWave;
    const uint32_t wave_first = (uint32_t)wave * quarter;
    const uint32_t wave_end = wave_first + quarter < gridDim.x ? wave_first + quarter : gridDim.x;
    C result = COp::identity();
    SpinState sp{0u, a.spin_limit, a.abort_flag, a.call_seq};
    bool ok = true;
    for (uint32_t base = wave_first; base < wave_end && ok; base += kFinishWindows * kWave) {
        C val[kFinishWindows];
        uint32_t st[kFinishWindows];
#pragma unroll
        for (int k = 0; k < kFinishWindows; ++k) {
            val[k] = COp::identity();
            st[k] = base + k * kWave + lane < wave_end ? kUnset : kPartial;   // nothing there: an empty partial
        }
        for (;;) {
            bool unset = false;
#pragma unroll
            for (int k = 0; k < kFinishWindows; ++k) {
                if (st[k] == kUnset) st[k] = desc_read<C>(a.partials, base + k * kWave + lane, a.epoch, val[k]);
                unset = unset || st[k] == kUnset;
            }
            if (__ballot(unset) == 0) break;
            if (!spin_once(sp)) {
                ok = false;
                break;
            }
        }
#pragma unroll
        for (int k = 0; k < kFinishWindows; ++k) {
            if (base + k * kWave + lane >= wave_end) val[k] = COp::identity();
            result = cop(result, read_lane(wave_inclusive_scan(val[k], cop), kWave - 1));
        }
    }
    if (lane == 0) {
        s_tot[wave] = to_words(result);
        if (!ok) s_last = 2u;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_last == 1u) {
            C total = from_words<C>(s_tot[0]);
#pragma unroll
            for (int k = 1; k < kWaves; ++k) total = cop(total, from_words<C>(s_tot[k]));
            if constexpr (ResultOf<Op, IO>::from_map) out[0] = convert<R>(total);   // f: T -> S, the result is an S
            else out[0] = convert<IO>(convert<A>(total));
        }
        reset_arrivals(a.control);   // ready for the next call
    }
}

}  // namespace ks
