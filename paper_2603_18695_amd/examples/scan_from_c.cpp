// The C ABI from a program of its own, without Python: an exclusive sum scan of uint32_t (the offsets of
// a stream compaction, paper Sec. II-C) and the single-launch reduction of the same array, both checked
// against a loop on the host, then timed.
//
//   hipcc -O2 --offload-arch=gfx950 -I../../include scan_from_c.cpp -L.. -lks_scan -Wl,-rpath,'$ORIGIN/..' -o scan_from_c
//   ./scan_from_c [n]
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ks_scan.h"

#define HIP_OK(call)                                                                                  \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) {                                                                       \
            std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                    \
            return 2;                                                                                 \
        }                                                                                             \
    } while (0)
#define KS_OK_OR_FAIL(call)                                                                           \
    do {                                                                                              \
        int s_ = (call);                                                                              \
        if (s_ != KS_OK) {                                                                            \
            std::fprintf(stderr, "%s failed: %s (hip error %d)\n", #call, ks_status_string(s_), ks_last_hip_error()); \
            return 2;                                                                                 \
        }                                                                                             \
    } while (0)

int main(int argc, char **argv) {
    const size_t n = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : (size_t)50000003;
    std::vector<uint32_t> host(n), want(n), got(n);
    uint32_t state = 12345u, running = 0;
    for (size_t i = 0; i < n; ++i) {
        state = state * 1664525u + 1013904223u;          // flags of a compaction: about one element in three is kept
        host[i] = (state >> 16) % 3u == 0u;
        want[i] = running;                               // exclusive: out[0] is the identity
        running += host[i];
    }
    uint32_t *in = nullptr, *out = nullptr, *total = nullptr;
    HIP_OK(hipMalloc(&in, n * sizeof(uint32_t)));
    HIP_OK(hipMalloc(&out, n * sizeof(uint32_t)));
    HIP_OK(hipMalloc(&total, sizeof(uint32_t)));
    HIP_OK(hipMemcpy(in, host.data(), n * sizeof(uint32_t), hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    KS_OK_OR_FAIL(ks_scan(KS_U32, KS_SUM, /*inclusive=*/0, in, out, n, stream));
    KS_OK_OR_FAIL(ks_mapreduce(KS_U32, KS_MAP_IDENTITY, KS_SUM, in, n, total, stream));
    KS_OK_OR_FAIL(ks_scan_check(stream));                // waits for the stream; reports an abandoned wait
    uint32_t kept = 0;
    HIP_OK(hipMemcpy(got.data(), out, n * sizeof(uint32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&kept, total, sizeof(uint32_t), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < n; ++i) {
        if (got[i] != want[i]) {
            std::fprintf(stderr, "mismatch at %zu: %u != %u\n", i, got[i], want[i]);
            return 1;
        }
    }
    if (kept != running) {
        std::fprintf(stderr, "reduction %u != %u\n", kept, running);
        return 1;
    }

    const int reps = 50;
    for (int i = 0; i < 5; ++i) KS_OK_OR_FAIL(ks_scan(KS_U32, KS_SUM, 0, in, out, n, stream));
    HIP_OK(hipStreamSynchronize(stream));
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0; i < reps; ++i) KS_OK_OR_FAIL(ks_scan(KS_U32, KS_SUM, 0, in, out, n, stream));
    HIP_OK(hipStreamSynchronize(stream));
    const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() / reps;
    std::printf("%s: n = %zu, %u kept; exclusive scan and reduction match the host; scan %.1f us per call, %.0f GB/s\n",
                ks_version(), n, kept, us, 2.0 * n * sizeof(uint32_t) / us / 1e3);
    KS_OK_OR_FAIL(ks_release_scratch(stream));
    HIP_OK(hipStreamDestroy(stream));
    HIP_OK(hipFree(in));
    HIP_OK(hipFree(out));
    HIP_OK(hipFree(total));
    return 0;
}
