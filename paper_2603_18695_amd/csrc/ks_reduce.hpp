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
//     CONTIGUOUS range of runs in order (one ordered DPP reduction per row), and since the
//     partials are combined in workgroup order the result is the left fold: operators that do
//     not commute are served too, which the paper's strided accumulation cannot do.
//   - No designated workgroup that spins on flags: the workgroup that arrives LAST (a counter
//     in the scratch) folds the partials, so nobody waits for a workgroup that has not run.
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
    uint32_t *control;     // control block of the scratch; word 1 counts the workgroups that have published
    uint64_t *partials;    // gridDim.x entries of tagged words
    uint32_t epoch, spin_limit;
    uint32_t *abort_flag;
    uint32_t call_seq;
    uint32_t runs_per_wave;   // ordered (non-commutative) operators: contiguous runs per wave
    uint32_t head_skip;       // elements narrower than a dword: `in` was moved down to a dword boundary,
                              // and this many leading bytes of run 0 are not part of the input
};

constexpr int kFinishWindows = 4;   // windows of 64 partials a finishing wave has in flight at once

template <class IO, class Op, int ROWS>
__global__ __launch_bounds__(kBlock) void mapreduce_kernel(const IO *in, typename ResultOf<Op, IO>::type *out,
                                                           ReduceArgs a) {
    using A = typename Op::acc;
    using R = typename ResultOf<Op, IO>::type;
    using C = typename ChainOf<Op>::type;
    using COp = typename ChainOf<Op>::op;
    using S = TileShape<IO, ROWS>;
    constexpr size_t RUN = S::WAVE_ELEMS;
    __shared__ typename WordsOf<C>::type s_tot[kWaves];
    __shared__ uint32_t s_last;
    Op op;
    COp cop;
    const int lane = threadIdx.x & (kWave - 1);
    // uniform for the compiler too: the runs' buffer descriptors then stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane_bytes = lane * 16;
    const size_t gw = (size_t)blockIdx.x * kWaves + wave;
    // commutative: runs gw, gw + W, gw + 2W, ... (W = waves of the grid); ordered: a contiguous range
    const size_t step = Op::commutative ? (size_t)gridDim.x * kWaves : 1;
    size_t run = Op::commutative ? gw : gw * a.runs_per_wave;
    size_t end = Op::commutative ? a.total_runs : run + a.runs_per_wave;
    if (end > a.total_runs) end = a.total_runs;

    // Commutative: acc is the lane's own running value.  Otherwise: the wave's, the same in every lane.
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
        ThreadItems<A, ROWS, S::G> it;
        unpack_items<IO, ROWS, Op, false>(raw, lane_bytes, w.valid_bytes, (run + 1) * RUN > a.n, it);
        if constexpr (sizeof(IO) < 4) {
            if (run == 0 && a.head_skip != 0) {   // the bytes in front of the caller's first element
#pragma unroll
                for (int k = 0; k < S::G; ++k)
                    if (lane_bytes + k * (int)sizeof(IO) < (int)a.head_skip) it.x[0][k] = Op::identity();
            }
        }
        if constexpr (Op::commutative) {
            A mine = it.x[0][0];
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
#pragma unroll
                for (int k = 0; k < S::G; ++k)
                    if (j != 0 || k != 0) mine = op(mine, it.x[j][k]);
            }
            acc = cop(acc, convert<C>(mine));
        } else {
            A run_total = Op::identity();
#pragma unroll
            for (int j = 0; j < ROWS; ++j) {
                A g = it.x[j][0];
#pragma unroll
                for (int k = 1; k < S::G; ++k) g = op(g, it.x[j][k]);
                const A row_total = read_lane(wave_inclusive_scan(g, op), kWave - 1);   // lanes in order
                run_total = (j == 0) ? row_total : op(run_total, row_total);
            }
            acc = cop(acc, convert<C>(run_total));
        }
        if (run + step < end) {
            raw = nxt;
            w = wn;
        }
    }
    if constexpr (Op::commutative) acc = read_lane(wave_inclusive_scan(acc, cop), kWave - 1);
    if (lane == 0) s_tot[wave] = to_words(acc);
    __syncthreads();
    if (threadIdx.x == 0) {
        C partial = from_words<C>(s_tot[0]);
#pragma unroll
        for (int k = 1; k < kWaves; ++k) partial = cop(partial, from_words<C>(s_tot[k]));
        desc_publish<C>(a.partials, blockIdx.x, a.epoch, kPartial, partial);
        const uint32_t before = __hip_atomic_fetch_add(&a.control[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = before + 1u == gridDim.x ? 1u : 0u;
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
        __hip_atomic_store(&a.control[1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }
}

}  // namespace ks
