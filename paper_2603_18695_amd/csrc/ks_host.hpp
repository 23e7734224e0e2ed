// Host-side plumbing shared by the translation units of the library: the
// per-pair launch table, launch arguments and tuning options.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ks_scan.h"

namespace ks {

struct Options {
    long long spin_limit = 1ll << 20;
    long long wgs_per_cu = 0;     // 0 = occupancy query
    long long waves = 0;          // 0 = default for the type, else 4, 8 or 16 waves per workgroup
    long long rows = 0;           // 0 = default for the type, else 4, 8, 9, 12 or 16
    long long prefetch = -1;      // -1 = default, 0 / 1 forced
    long long form = -1;          // -1 = default, else 0 common loop, 1 separate loops, 2 separate + blocked,
                                  // 3 common loop with pauses, 4 / 5 = 0 / 3 with tiles on the output's
                                  // 128-byte lines (1-5: 16 waves only; 3-5: 9 rows with prefetch only)
    long long grid_mode = 0;      // 0 = persistent resident grid, 1 = one workgroup per tile (experimental)
    long long last_grid = 0;      // read-only: workgroups of the most recent look-back launch
    long long last_resident_per_cu = 0;   // read-only: verified resident workgroups per CU of that kernel variant
    long long last_waves = 0, last_rows = 0, last_form = 0;   // read-only: shape and form of that launch
};
Options &options();

struct DeviceInfo {
    int device = -1;
    int cus = 0;
    uint32_t *abort_flag = nullptr;   // device address of the library's abort word on this device
    uint32_t *residency = nullptr;    // two words used by the one-off residency check of a kernel variant
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
    bool clear_descriptors; // scratch contents unknown: zero the descriptors first
    const DeviceInfo *dev;
    // strided views (paper Sec. IV-C): element i at in[i * in_stride] / out[i * out_stride]; always
    // the look-back algorithm, temp as for it
    size_t in_stride = 1, out_stride = 1;
};

// One entry per instantiated (dtype, op) pair.
struct PairEntry {
    size_t elem_bytes;
    size_t elem_align;
    size_t (*temp_bytes)(ks_algo algo, size_t n);
    ks_algo (*pick_algo)(size_t n);
    int (*run)(const ScanCall &call);   // returns ks_status; HIP failures via set_hip_error
};

int set_hip_error(hipError_t e);   // records e, returns KS_ERR_HIP

// defined in the ks_pairs_*.hip files
const PairEntry *pair_entry(int dtype, int op);

}  // namespace ks
