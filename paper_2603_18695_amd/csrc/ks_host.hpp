// Host-side plumbing shared by the translation units of the library: the
// per-pair launch table, launch arguments and tuning options.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ks_scan.h"

namespace ks {

// Process-wide tuning options.  Read and written under the library's mutex (every entry point that
// launches holds it), so a change never lands in the middle of a launch.
struct Options {
    long long spin_limit = 1ll << 20;
    long long wgs_per_cu = 0;     // 0 = what the occupancy query gives, else 1 .. 64
    long long waves = 0;          // 0 = default for the type, else 4, 8 or 16 waves per workgroup
    long long rows = 0;           // 0 = default for the type, else 4, 8, 9, 12 or 16
    long long prefetch = -1;      // -1 = default, 0 / 1 forced
    long long form = -1;          // -1 = default, else 0 common loop (4 and 8 waves), 1 separate loops,
                                  // 2 separate loops + blocked arrangement (16 waves)
    long long tickets = -1;       // tile assignment: -1 = by index for grids of up to one workgroup per compute
                                  // unit, by ticket for larger ones; 1 = always by ticket
};
Options &options();

// What the calling thread's most recent look-back launch ran (read-only "last_*" options).
struct LastLaunch {
    long long grid = 0, wgs_per_cu = 0, waves = 0, rows = 0, form = 0, tickets = 0;
};
LastLaunch &last_launch();

struct DeviceInfo {
    int device = -1;
    int cus = 0;
    uint32_t *abort_table = nullptr;   // device address of the library's table of abort words on this device
    void *static_scratch = nullptr;    // device address of this device's copy of the static scratch array
};

struct ScanCall {
    int inclusive;
    ks_algo algo;           // never AUTO here
    const void *in;
    void *out;
    size_t n;
    void *temp;             // device scratch, 256-byte aligned
    size_t temp_bytes;
    hipStream_t stream;
    uint32_t epoch;         // tag for this call's descriptors (look-back only)
    bool clear_descriptors; // scratch contents unknown: zero control block and descriptors first
    const DeviceInfo *dev;
    uint32_t *abort_flag;   // abort word of the call's (device, stream)
    uint32_t call_seq;      // sequence number of the call on its stream, never zero
    // strided views (paper Sec. IV-C): element i at in[i * in_stride] / out[i * out_stride]; always
    // the look-back algorithm, temp as for it
    size_t in_stride = 1, out_stride = 1;
    // seeded scan: device pointer to one element that precedes in[0] (look-back algorithm, contiguous arrays)
    const void *seed = nullptr;
};

// One entry per instantiated (dtype, op) pair.  Pair<T, Op>::entry() may also be instantiated outside
// the library, in a translation unit of the caller's that includes ks_launch.hpp, for a type and an
// operator of the caller's (ks_scan_pair / ks_mapreduce_pair take the pointer); `abi` tells the
// library that both sides were compiled against the same layout of this struct and of ScanCall.
constexpr uint32_t kPairAbi = 0x4b530002u;
struct PairEntry {
    uint32_t abi;
    size_t elem_bytes;
    size_t elem_align;
    size_t (*temp_bytes)(ks_algo algo, size_t n);
    ks_algo (*pick_algo)(size_t n);
    int (*run)(const ScanCall &call);   // returns ks_status; HIP failures via set_hip_error
    int (*mapreduce)(const ScanCall &call);   // call.out = one element; call.temp = control block + partials
    size_t result_bytes, result_align;        // of what mapreduce writes (the map's result type)
    // temp_bytes, pick_algo and run are null for pairs that are only reduced (byte elements)
};

int set_hip_error(hipError_t e);   // records e, returns KS_ERR_HIP

// defined in the ks_pairs_*.hip files
const PairEntry *pair_entry(int dtype, int op);

}  // namespace ks
