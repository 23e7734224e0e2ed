// Two element types and operators defined OUTSIDE the library (paper Sec. IV-A: the primitives work
// for any struct of plain fields and any associative operator the caller writes).  Built by hipcc for
// gfx950 against the headers in ../csrc and linked with libks_scan.so; the entry points below hand the
// pairs to ks_scan_pair / ks_mapreduce_pair (include/ks_scan.h).
//
//   hipcc -O3 -std=c++17 --offload-arch=gfx950 -fno-gpu-rdc -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -fPIC -shared -I../csrc user_pair.hip -L.. -lks_scan -Wl,-rpath,'$ORIGIN/..' -o libks_user_pair.so
// (the flags the library itself is built with: build.py)
#include "ks_launch.hpp"

namespace {

// x -> a * x + b over Z/2^32 (8 bytes).  Composition is associative and does not commute: a scan
// of such maps solves the linear recurrence x_i = a_i * x_(i-1) + b_i exactly.
struct AffineU32 {
    uint32_t a, b;
};
struct AffineU32Compose {
    static constexpr bool commutative = false;
    using acc = AffineU32;
    __device__ static AffineU32 identity() { return AffineU32{1u, 0u}; }
    // first `earlier`, then `later`: later(earlier(x)) = later.a * (earlier.a * x + earlier.b) + later.b
    __device__ __forceinline__ AffineU32 operator()(AffineU32 earlier, AffineU32 later) const {
        return AffineU32{later.a * earlier.a, later.a * earlier.b + later.b};
    }
};

// Running statistics of a stream of int32 samples (24 bytes: neither 4, 8 nor 16, so the kernels take
// the arrangement in which a lane holds 9 consecutive 16-byte granules = 6 elements).
struct Stats24 {
    int64_t sum;     // wraps modulo 2^64
    int32_t lo, hi;  // smallest and largest sample
    uint64_t cnt;    // number of samples
};
struct Stats24Merge {
    static constexpr bool commutative = true;
    using acc = Stats24;
    __device__ static Stats24 identity() { return Stats24{0, INT32_MAX, INT32_MIN, 0ull}; }
    __device__ __forceinline__ Stats24 operator()(Stats24 l, Stats24 r) const {
        return Stats24{(int64_t)((uint64_t)l.sum + (uint64_t)r.sum), l.lo < r.lo ? l.lo : r.lo, l.hi > r.hi ? l.hi : r.hi,
                       l.cnt + r.cnt};
    }
};

}  // namespace

extern "C" const void *ks_user_affine_u32_pair() { return ks::Pair<AffineU32, AffineU32Compose>::entry(); }
extern "C" const void *ks_user_stats24_pair() { return ks::Pair<Stats24, Stats24Merge>::entry(); }
