// C ABI of the scan library: argument validation, (dtype, op) lookup, the
// library-owned workspace cache and the status / option entry points.
// Declarations and conventions: include/ks_scan.h.
#include <hip/hip_runtime.h>

#include <cstring>
#include <map>
#include <mutex>
#include <utility>

#include "ks_host.hpp"
#include "ks_kernels.hpp"

namespace ks {

// Abort words: one per (device, stream) that has run a look-back scan, handed out in order of first
// use.  A look-back wave that exhausts its spin limit writes its call's sequence number there.
// Static device memory, so that handing out a slot allocates nothing.
constexpr int kAbortSlots = 1024;
__device__ uint32_t g_abort_table[kAbortSlots];

// Scratch of ks_scan_static: device memory that exists without any allocation call.  One array per
// device that loads the library; host code reaches it through the address hipGetSymbolAddress
// returns for the current device (DeviceInfo::static_scratch), never through this name.
constexpr size_t kStaticScratchBytes = (size_t)KS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

const PairEntry *pair_entry_i32(int, int);
const PairEntry *pair_entry_i64(int, int);
const PairEntry *pair_entry_float(int, int);
const PairEntry *pair_entry_struct(int, int);
const PairEntry *pair_entry_mapped(int, int, int);
const PairEntry *pair_entry_bytes(int, int, int);
const PairEntry *pair_entry_half(int, int);

const PairEntry *pair_entry(int dtype, int op) {
    if (dtype < 0 || dtype >= KS_DTYPE_COUNT || op < 0 || op >= KS_OP_COUNT) return nullptr;
    if (const PairEntry *e = pair_entry_i32(dtype, op)) return e;
    if (const PairEntry *e = pair_entry_i64(dtype, op)) return e;
    if (const PairEntry *e = pair_entry_float(dtype, op)) return e;
    if (const PairEntry *e = pair_entry_half(dtype, op)) return e;
    return pair_entry_struct(dtype, op);
}

Options &options() {
    static Options o;
    return o;
}
LastLaunch &last_launch() {
    static thread_local LastLaunch l;
    return l;
}

static thread_local int t_last_hip = 0;
int set_hip_error(hipError_t e) {
    t_last_hip = (int)e;
    return KS_ERR_HIP;
}

namespace {

std::mutex g_mutex;
std::map<int, DeviceInfo> g_devices;

// Per (device, stream): the library-owned scratch of ks_scan, the stream's abort word and the
// sequence number of its calls.
struct StreamState {
    void *ptr = nullptr;
    size_t bytes = 0;
    uint32_t epoch = 0;       // last epoch handed out; descriptors carry (epoch << 2 | state)
    bool captured = false;    // a stream capture has recorded a call that uses ptr: never freed again
    int abort_slot = -1;
    uint32_t seq = 0;         // sequence number of the last call; the next one takes seq + 1 (never zero)
};
std::map<std::pair<int, hipStream_t>, StreamState> g_streams;
int g_next_abort_slot[64] = {0};   // per device

// Epochs 1 .. kMaxEagerEpoch tag ordinary calls; a call recorded into a graph clears its
// descriptors itself and uses kCaptureEpoch, which no ordinary call ever carries.
constexpr uint32_t kCaptureEpoch = (1u << 30) - 1;
constexpr uint32_t kMaxEagerEpoch = kCaptureEpoch - 1;

int device_info(const DeviceInfo **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_hip_error(e);
    auto it = g_devices.find(dev);
    if (it == g_devices.end()) {
        DeviceInfo d;
        d.device = dev;
        e = hipDeviceGetAttribute(&d.cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return set_hip_error(e);
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_abort_table));
        if (e != hipSuccess) return set_hip_error(e);
        d.abort_table = static_cast<uint32_t *>(p);
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return set_hip_error(e);
        d.static_scratch = p;
        it = g_devices.emplace(dev, d).first;
    }
    *out = &it->second;
    return KS_OK;
}

// The stream's state, with an abort word assigned and the next sequence number taken.
StreamState &stream_state(const DeviceInfo *dev, hipStream_t stream) {
    StreamState &st = g_streams[std::make_pair(dev->device, stream)];
    if (st.abort_slot < 0) {
        int &next = g_next_abort_slot[dev->device & 63];
        st.abort_slot = next % kAbortSlots;   // more streams than slots: the oldest slots are shared
        ++next;
    }
    if (++st.seq == 0) st.seq = 1;
    return st;
}

// pointers, size and overlap of a scan's arguments for the pair `e`
int validate_arrays(const PairEntry *e, const void *in, void *out, size_t n);

int validate(ks_dtype dtype, ks_op op, const void *in, void *out, size_t n, const PairEntry **entry) {
    if ((int)dtype < 0 || dtype >= KS_DTYPE_COUNT || (int)op < 0 || op >= KS_OP_COUNT) return KS_ERR_INVALID_ARG;
    const PairEntry *e = pair_entry(dtype, op);
    if (!e || !e->run) return KS_ERR_UNSUPPORTED;
    *entry = e;
    return validate_arrays(e, in, out, n);
}

int validate_arrays(const PairEntry *e, const void *in, void *out, size_t n) {
    if (n == 0) return KS_OK;
    if (!in || !out) return KS_ERR_INVALID_ARG;
    if (n > ((size_t)1 << 40)) return KS_ERR_INVALID_ARG;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if ((a % e->elem_align) || (b % e->elem_align)) return KS_ERR_MISALIGNED;
    const size_t bytes = n * e->elem_bytes;
    if (a != b && a < b + bytes && b < a + bytes) return KS_ERR_OVERLAP;
    return KS_OK;
}

}  // namespace
}  // namespace ks

using namespace ks;

extern "C" {

int ks_scan_with_temp(ks_dtype dtype, ks_op op, int inclusive, ks_algo algo, const void *in, void *out, size_t n,
                      void *temp, size_t temp_bytes, void *stream) {
    const PairEntry *e = nullptr;
    int st = validate(dtype, op, in, out, n, &e);
    if (st != KS_OK || n == 0) return st;
    if ((int)algo < KS_ALGO_AUTO || (int)algo > KS_ALGO_REDUCE_THEN_SCAN) return KS_ERR_INVALID_ARG;
    if (algo == KS_ALGO_AUTO) algo = e->pick_algo(n);
    if (!temp || ((uintptr_t)temp & 255u) || temp_bytes < e->temp_bytes(algo, n)) return KS_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_mutex);
    const DeviceInfo *dev = nullptr;
    if ((st = device_info(&dev)) != KS_OK) return st;
    StreamState &ss = stream_state(dev, (hipStream_t)stream);
    ScanCall c{inclusive, algo, in, out, n, temp, temp_bytes, (hipStream_t)stream, 1u, true, dev,
               dev->abort_table + ss.abort_slot, ss.seq};
    return e->run(c);
}

// Common part of ks_scan, ks_scan_map and ks_scan_strided: library-owned, epoch-tagged scratch per
// (device, stream).  Strided views always take the look-back algorithm.
static int scan_with_library_workspace(const PairEntry *e, int inclusive, const void *in, void *out, size_t n,
                                       void *stream, size_t in_stride = 1, size_t out_stride = 1,
                                       bool reduce = false, const void *seed = nullptr) {
    const bool strided = in_stride != 1 || out_stride != 1;
    // strided views, reductions and seeded scans always take the single-pass route (all tag their scratch with an epoch)
    const ks_algo algo = strided || reduce || seed ? KS_ALGO_LOOKBACK : e->pick_algo(n);
    // a reduction's scratch (control block and one partial per workgroup) always fits the smallest buffer
    const size_t need = reduce ? 1 : e->temp_bytes(algo, n);
    std::lock_guard<std::mutex> lock(g_mutex);
    const DeviceInfo *dev = nullptr;
    int st;
    if ((st = device_info(&dev)) != KS_OK) return st;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    hipError_t he = hipStreamIsCapturing((hipStream_t)stream, &capture);
    if (he != hipSuccess) return set_hip_error(he);
    const bool capturing = capture != hipStreamCaptureStatusNone;
    StreamState &ws = stream_state(dev, (hipStream_t)stream);
    bool fresh = false;
    if (ws.bytes < need) {
        if (capturing) return KS_ERR_WORKSPACE;   // no allocation under capture: make a larger eager call first
        // growing: hipFree waits for the device, so nothing in flight still uses the old buffer.  A
        // buffer that a graph has recorded stays allocated for good: the graph may be replayed.
        if (ws.ptr && !ws.captured) (void)hipFree(ws.ptr);
        ws.ptr = nullptr;
        ws.bytes = 0;
        ws.captured = false;
        const size_t want = need < ((size_t)1 << 20) ? ((size_t)1 << 20) : need;
        he = hipMalloc(&ws.ptr, want);
        if (he != hipSuccess) {
            ws.ptr = nullptr;
            set_hip_error(he);
            return KS_ERR_WORKSPACE;
        }
        ws.bytes = want;
        fresh = true;
    }
    uint32_t epoch = 0;
    bool clear = false;
    if (capturing) {
        // A graph replays the same kernel arguments every time, so the epoch cannot tell a replay's
        // descriptors from those of the replay before: the recorded call clears its scratch itself
        // (with a kernel) and carries an epoch of its own.
        ws.captured = true;
        epoch = kCaptureEpoch;
        clear = true;
    } else {
        if (fresh || ws.epoch >= kMaxEagerEpoch) {
            // a fill kernel, not hipMemsetAsync: memset nodes misbehave in graphs on this platform, and
            // one code path for both is simpler
            const size_t words = ws.bytes / sizeof(uint64_t);
            const size_t blocks = (words + 255) / 256;
            hipLaunchKernelGGL((fill_zero_kernel<0>), dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0,
                               (hipStream_t)stream, static_cast<uint64_t *>(ws.ptr), words);
            he = hipGetLastError();
            if (he != hipSuccess) return set_hip_error(he);
            ws.epoch = 0;
        }
        if (algo == KS_ALGO_LOOKBACK) ++ws.epoch;
        epoch = ws.epoch;
    }
    ScanCall c{inclusive, algo, in, out, n, ws.ptr, ws.bytes, (hipStream_t)stream, epoch, clear, dev,
               dev->abort_table + ws.abort_slot, ws.seq, in_stride, out_stride, seed};
    return reduce ? e->mapreduce(c) : e->run(c);
}

int ks_scan(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n, void *stream) {
    const PairEntry *e = nullptr;
    int st = validate(dtype, op, in, out, n, &e);
    if (st != KS_OK || n == 0) return st;
    return scan_with_library_workspace(e, inclusive, in, out, n, stream);
}

int ks_scan_seeded(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n, const void *seed,
                   void *stream) {
    const PairEntry *e = nullptr;
    int st = validate(dtype, op, in, out, n, &e);
    if (st != KS_OK || n == 0) return st;
    if (!seed) return KS_ERR_INVALID_ARG;
    if ((uintptr_t)seed % (e->elem_bytes < 4 ? e->elem_bytes : e->elem_align)) return KS_ERR_MISALIGNED;
    return scan_with_library_workspace(e, inclusive, in, out, n, stream, 1, 1, false, seed);
}

int ks_scan_static(ks_dtype dtype, ks_op op, int inclusive, const void *in, void *out, size_t n, void *stream) {
    const PairEntry *e = nullptr;
    int st = validate(dtype, op, in, out, n, &e);
    if (st != KS_OK || n == 0) return st;
    const ks_algo algo = e->pick_algo(n);
    if (e->temp_bytes(algo, n) > kStaticScratchBytes) return KS_ERR_WORKSPACE;   // beyond the stated maximum
    std::lock_guard<std::mutex> lock(g_mutex);
    const DeviceInfo *dev = nullptr;
    if ((st = device_info(&dev)) != KS_OK) return st;
    StreamState &ss = stream_state(dev, (hipStream_t)stream);
    // the array keeps what the last call left: the launch code clears what this call uses, with a kernel
    ScanCall c{inclusive, algo, in, out, n, dev->static_scratch, kStaticScratchBytes, (hipStream_t)stream, 1u, true,
               dev, dev->abort_table + ss.abort_slot, ss.seq};
    return e->run(c);
}

int ks_scan_map(ks_dtype dtype, ks_map map, ks_op op, int inclusive, const void *in, void *out, size_t n,
                void *stream) {
    if (map == KS_MAP_IDENTITY) return ks_scan(dtype, op, inclusive, in, out, n, stream);
    const PairEntry *plain = nullptr;
    int st = validate(dtype, op, in, out, n, &plain);   // pointers, alignment, overlap: as for the plain pair
    if (st != KS_OK) return st;
    const PairEntry *e = pair_entry_mapped((int)dtype, (int)map, (int)op);
    if (!e) return KS_ERR_UNSUPPORTED;
    if (n == 0) return KS_OK;
    return scan_with_library_workspace(e, inclusive, in, out, n, stream);
}

int ks_scan_strided(ks_dtype dtype, ks_op op, int inclusive, const void *in, size_t in_stride, void *out,
                    size_t out_stride, size_t n, void *stream) {
    if (in_stride == 1 && out_stride == 1) return ks_scan(dtype, op, inclusive, in, out, n, stream);
    if ((int)dtype < 0 || dtype >= KS_DTYPE_COUNT || (int)op < 0 || op >= KS_OP_COUNT) return KS_ERR_INVALID_ARG;
    const PairEntry *e = pair_entry(dtype, op);
    if (!e) return KS_ERR_UNSUPPORTED;
    if (n == 0) return KS_OK;
    if (!in || !out || in_stride == 0 || out_stride == 0) return KS_ERR_INVALID_ARG;
    if (n > ((size_t)1 << 40) || in_stride > ((size_t)1 << 20) || out_stride > ((size_t)1 << 20)) return KS_ERR_INVALID_ARG;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if ((a % e->elem_align) || (b % e->elem_align)) return KS_ERR_MISALIGNED;
    // byte spans of the two views; the same view in place is fine, any other overlap of the spans is refused
    const size_t span_in = ((n - 1) * in_stride + 1) * e->elem_bytes, span_out = ((n - 1) * out_stride + 1) * e->elem_bytes;
    const bool same_view = a == b && in_stride == out_stride;
    if (!same_view && a < b + span_out && b < a + span_in) return KS_ERR_OVERLAP;
    return scan_with_library_workspace(e, inclusive, in, out, n, stream, in_stride, out_stride);
}

// the entry whose mapreduce serves (dtype, map, op), or null
static const PairEntry *reduce_entry(int dtype, int map, int op) {
    if (dtype < 0 || dtype >= KS_DTYPE_COUNT || op < 0 || op >= KS_OP_COUNT || map < 0 || map >= KS_MAP_COUNT)
        return nullptr;
    if (dtype == KS_U8 || dtype == KS_BF16 || dtype == KS_F16) return pair_entry_bytes(dtype, map, op);
    return map == KS_MAP_IDENTITY ? pair_entry(dtype, op) : pair_entry_mapped(dtype, map, op);
}

int ks_mapreduce(ks_dtype dtype, ks_map map, ks_op op, const void *in, size_t n, void *out, void *stream) {
    if ((int)dtype < 0 || dtype >= KS_DTYPE_COUNT || (int)op < 0 || op >= KS_OP_COUNT) return KS_ERR_INVALID_ARG;
    if ((int)map < KS_MAP_IDENTITY || (int)map >= KS_MAP_COUNT) return KS_ERR_INVALID_ARG;
    const PairEntry *e = reduce_entry((int)dtype, (int)map, (int)op);
    if (!e) return KS_ERR_UNSUPPORTED;
    if (!out || (n > 0 && !in)) return KS_ERR_INVALID_ARG;
    if (n > ((size_t)1 << 40)) return KS_ERR_INVALID_ARG;
    if (((uintptr_t)in % e->elem_align) || ((uintptr_t)out % e->result_align)) return KS_ERR_MISALIGNED;
    return scan_with_library_workspace(e, 1, in, out, n, stream, 1, 1, true);
}

size_t ks_mapreduce_result_bytes(ks_dtype dtype, ks_map map, ks_op op) {
    const PairEntry *e = reduce_entry((int)dtype, (int)map, (int)op);
    return e ? e->result_bytes : 0;
}

// A pair compiled by the caller: the pointer must be what Pair<T, Op>::entry() returned to code
// built against this version of the library's headers.
static const PairEntry *caller_pair(const void *pair) {
    const PairEntry *e = static_cast<const PairEntry *>(pair);
    return e && e->abi == kPairAbi ? e : nullptr;
}

int ks_scan_pair(const void *pair, int inclusive, const void *in, void *out, size_t n, void *stream) {
    const PairEntry *e = caller_pair(pair);
    if (!e) return KS_ERR_INVALID_ARG;
    if (!e->run) return KS_ERR_UNSUPPORTED;
    const int st = validate_arrays(e, in, out, n);
    if (st != KS_OK || n == 0) return st;
    return scan_with_library_workspace(e, inclusive, in, out, n, stream);
}

int ks_mapreduce_pair(const void *pair, const void *in, size_t n, void *out, void *stream) {
    const PairEntry *e = caller_pair(pair);
    if (!e) return KS_ERR_INVALID_ARG;
    if (!e->mapreduce) return KS_ERR_UNSUPPORTED;
    if (!out || (n > 0 && !in)) return KS_ERR_INVALID_ARG;
    if (n > ((size_t)1 << 40)) return KS_ERR_INVALID_ARG;
    if (((uintptr_t)in % e->elem_align) || ((uintptr_t)out % e->result_align)) return KS_ERR_MISALIGNED;
    return scan_with_library_workspace(e, 1, in, out, n, stream, 1, 1, true);
}

size_t ks_pair_elem_bytes(const void *pair) {
    const PairEntry *e = caller_pair(pair);
    return e ? e->elem_bytes : 0;
}

int ks_release_scratch(void *stream) {
    hipError_t he = hipStreamSynchronize((hipStream_t)stream);   // nothing in flight may still use the buffer
    if (he != hipSuccess) return set_hip_error(he);
    std::lock_guard<std::mutex> lock(g_mutex);
    const DeviceInfo *dev = nullptr;
    int st;
    if ((st = device_info(&dev)) != KS_OK) return st;
    auto it = g_streams.find(std::make_pair(dev->device, (hipStream_t)stream));
    if (it == g_streams.end()) return KS_OK;
    StreamState &ws = it->second;
    if (!ws.ptr || ws.captured) return KS_OK;   // nothing cached, or a graph may still replay into it
    he = hipFree(ws.ptr);
    ws.ptr = nullptr;
    ws.bytes = 0;
    ws.epoch = 0;
    return he == hipSuccess ? KS_OK : set_hip_error(he);
}

int ks_map_supported(ks_dtype dtype, ks_map map, ks_op op) {
    if (map == KS_MAP_IDENTITY) return ks_pair_supported(dtype, op);
    return pair_entry_mapped((int)dtype, (int)map, (int)op) ? 1 : 0;
}

size_t ks_scan_temp_bytes(ks_dtype dtype, ks_op op, ks_algo algo, size_t n) {
    const PairEntry *e = pair_entry((int)dtype, (int)op);
    if (!e || (int)algo < KS_ALGO_AUTO || (int)algo > KS_ALGO_REDUCE_THEN_SCAN) return 0;
    return e->temp_bytes(algo, n);
}

int ks_scan_check(void *stream) {
    hipError_t he = hipStreamSynchronize((hipStream_t)stream);
    if (he != hipSuccess) return set_hip_error(he);
    std::lock_guard<std::mutex> lock(g_mutex);
    const DeviceInfo *dev = nullptr;
    int st;
    if ((st = device_info(&dev)) != KS_OK) return st;
    auto it = g_streams.find(std::make_pair(dev->device, (hipStream_t)stream));
    if (it == g_streams.end() || it->second.abort_slot < 0) return KS_OK;   // no scan has run on this stream
    uint32_t *word = dev->abort_table + it->second.abort_slot;
    uint32_t flag = 0;
    he = hipMemcpy(&flag, word, sizeof(flag), hipMemcpyDeviceToHost);
    if (he != hipSuccess) return set_hip_error(he);
    if (flag != 0) {
        const uint32_t zero = 0;
        he = hipMemcpy(word, &zero, sizeof(zero), hipMemcpyHostToDevice);
        if (he != hipSuccess) return set_hip_error(he);
        return KS_ERR_TIMEOUT;
    }
    return KS_OK;
}

int ks_pair_supported(ks_dtype dtype, ks_op op) { return pair_entry((int)dtype, (int)op) ? 1 : 0; }

size_t ks_elem_bytes(ks_dtype dtype) {
    switch (dtype) {
        case KS_I32: case KS_U32: case KS_F32: return 4;
        case KS_I64: case KS_U64: case KS_F64: case KS_AFFINE_F32: return 8;
        case KS_ARGMAX_I32_CNT64: case KS_MAT2_U32: case KS_QUAT_F32: return 16;
        case KS_MAT2_U64: return 32;
        case KS_RANGE_I32_CNT32: return 12;
        case KS_U8: return 1;
        case KS_BF16: case KS_F16: return 2;
        default: return 0;
    }
}

static long long *option_slot(const char *name) {
    if (!name) return nullptr;
    Options &o = options();
    if (!std::strcmp(name, "spin_limit")) return &o.spin_limit;
    if (!std::strcmp(name, "wgs_per_cu")) return &o.wgs_per_cu;
    if (!std::strcmp(name, "rows")) return &o.rows;
    if (!std::strcmp(name, "waves")) return &o.waves;
    if (!std::strcmp(name, "prefetch")) return &o.prefetch;
    if (!std::strcmp(name, "form")) return &o.form;
    if (!std::strcmp(name, "tickets")) return &o.tickets;
    return nullptr;
}

static const long long *last_slot(const char *name) {
    if (!name) return nullptr;
    const LastLaunch &l = last_launch();
    if (!std::strcmp(name, "last_grid")) return &l.grid;
    if (!std::strcmp(name, "last_wgs_per_cu")) return &l.wgs_per_cu;
    if (!std::strcmp(name, "last_waves")) return &l.waves;
    if (!std::strcmp(name, "last_rows")) return &l.rows;
    if (!std::strcmp(name, "last_form")) return &l.form;
    if (!std::strcmp(name, "last_tickets")) return &l.tickets;
    return nullptr;
}

int ks_set_option(const char *name, long long value) {
    std::lock_guard<std::mutex> lock(g_mutex);
    long long *slot = option_slot(name);
    if (!slot) return KS_ERR_INVALID_ARG;   // unknown, or one of the read-only "last_*" names
    Options &o = options();
    if (slot == &o.waves && !(value == 0 || value == 4 || value == 8 || value == 16)) return KS_ERR_INVALID_ARG;
    if (slot == &o.rows && !(value == 0 || value == 4 || value == 8 || value == 9 || value == 12 || value == 16)) return KS_ERR_INVALID_ARG;
    if (slot == &o.spin_limit && value < 0) return KS_ERR_INVALID_ARG;
    if (slot == &o.wgs_per_cu && (value < 0 || value > 64)) return KS_ERR_INVALID_ARG;
    if (slot == &o.prefetch && !(value >= -1 && value <= 1)) return KS_ERR_INVALID_ARG;
    if (slot == &o.form && !(value >= -1 && value < kFormCount)) return KS_ERR_INVALID_ARG;
    if (slot == &o.tickets && !(value == -1 || value == 1)) return KS_ERR_INVALID_ARG;
    *slot = value;
    return KS_OK;
}

long long ks_get_option(const char *name) {
    if (const long long *last = last_slot(name)) return *last;
    std::lock_guard<std::mutex> lock(g_mutex);
    long long *slot = option_slot(name);
    return slot ? *slot : -1;
}

int ks_copy(const void *in, void *out, size_t bytes, void *stream) {
    if (bytes == 0) return KS_OK;
    if (!in || !out) return KS_ERR_INVALID_ARG;
    if ((bytes & 15u) || ((uintptr_t)in & 15u) || ((uintptr_t)out & 15u)) return KS_ERR_MISALIGNED;
    const uintptr_t a = (uintptr_t)in, b = (uintptr_t)out;
    if (a < b + bytes && b < a + bytes) return KS_ERR_OVERLAP;
    // One granule per thread in 256-thread workgroups is the fastest plain copy found on MI355X
    // (2 x 1 GiB: 6.45 TB/s; 2 granules 6.1-6.4, 4 granules 6.3, 512- and 1024-thread workgroups
    // 5.8-6.3, persistent grid-stride grids 5.6-5.9, ordinary instead of non-temporal accesses 5.8).
    constexpr int ROWS = 1;
    const size_t granules = bytes / 16;
    const size_t per_wg = (size_t)kBlock * ROWS;
    const size_t grid = (granules + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffull) return KS_ERR_INVALID_ARG;
    hipLaunchKernelGGL((copy_kernel<ROWS>), dim3((unsigned)grid), dim3(kBlock), 0, (hipStream_t)stream,
                       static_cast<const u32x4 *>(in), static_cast<u32x4 *>(out), granules);
    hipError_t he = hipGetLastError();
    return he == hipSuccess ? KS_OK : set_hip_error(he);
}

const char *ks_status_string(int status) {
    switch (status) {
        case KS_OK: return "ok";
        case KS_ERR_INVALID_ARG: return "invalid argument";
        case KS_ERR_UNSUPPORTED: return "(dtype, op) pair not supported";
        case KS_ERR_MISALIGNED: return "pointer not aligned to the element type";
        case KS_ERR_OVERLAP: return "in and out overlap without being identical";
        case KS_ERR_WORKSPACE: return "scratch buffer missing, too small, misaligned or not allocatable";
        case KS_ERR_HIP: return "HIP runtime error (see ks_last_hip_error)";
        case KS_ERR_TIMEOUT: return "a look-back wait exceeded its spin limit";
        default: return "unknown status";
    }
}

int ks_last_hip_error(void) { return t_last_hip; }

const char *ks_version(void) { return "ks_scan 0.1 (gfx950)"; }

}  // extern "C"
