// Host time of one sgemm_tuned_on() call that hits the dispatch cache, measured from C beside
// the host time of a plain HIP launch of an empty kernel (the floor any launch pays).  The paper
// proposes tuning per input at run time ("CLTune: an auto-tuner for OpenCL kernels"), which
// makes the cost of finding the tuned variant on every call matter for small problems.
//
//   dispatch_overhead M N K layout [calls]
//
// Calls are issued in bursts of 32 with a stream synchronisation (untimed) between bursts, so
// that no call waits for room in the queue; each call is timed on its own with the steady
// clock.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/sgemm_tuned.h"

__global__ void empty_kernel(int) {}

static double median(std::vector<double> v) {
    std::sort(v.begin(), v.end());
    return v[v.size() / 2];
}

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                  \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)

int main(int argc, char **argv) {
    if (argc < 5) {
        std::fprintf(stderr, "usage: %s M N K layout [calls]\n", argv[0]);
        return 2;
    }
    const int M = std::atoi(argv[1]), N = std::atoi(argv[2]), K = std::atoi(argv[3]), layout = std::atoi(argv[4]);
    const int calls = argc > 5 ? std::atoi(argv[5]) : 4096;
    const int lda = (layout & 1) ? M : K, ldb = (layout & 2) ? K : N, ldc = N;
    float *A, *B, *C;
    CHECK(hipMalloc(&A, sizeof(float) * (size_t)M * K));
    CHECK(hipMalloc(&B, sizeof(float) * (size_t)K * N));
    CHECK(hipMalloc(&C, sizeof(float) * (size_t)M * N));
    CHECK(hipMemset(A, 0, sizeof(float) * (size_t)M * K));
    CHECK(hipMemset(B, 0, sizeof(float) * (size_t)K * N));
    hipStream_t s;
    CHECK(hipStreamCreate(&s));
    // first call: resolves, loads and plans (the slow half of the dispatch)
    auto t0 = std::chrono::steady_clock::now();
    int rc = sgemm_tuned_on(s, M, N, K, 1.0f, A, lda, B, ldb, 0.0f, C, ldc, layout);
    if (rc != SGEMM_OK) {
        std::fprintf(stderr, "sgemm_tuned_on: %s: %s\n", sgemm_status_string(rc), sgemm_last_error());
        return 1;
    }
    CHECK(hipStreamSynchronize(s));
    const double first_us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();

    std::vector<double> lib_us, raw_us;
    for (int pass = 0; pass < 2; ++pass) {
        std::vector<double> &out = pass == 0 ? raw_us : lib_us;
        for (int i = 0; i < calls + 64; ++i) { // the first 64 are warm-up
            const auto a = std::chrono::steady_clock::now();
            if (pass == 0) {
                hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s, 0);
            } else {
                rc = sgemm_tuned_on(s, M, N, K, 1.0f, A, lda, B, ldb, 0.0f, C, ldc, layout);
            }
            const auto b = std::chrono::steady_clock::now();
            if (rc != SGEMM_OK) return 1;
            if (i >= 64) out.push_back(std::chrono::duration<double, std::micro>(b - a).count());
            if (i % 32 == 31) CHECK(hipStreamSynchronize(s));
        }
        CHECK(hipStreamSynchronize(s));
    }
    const double lib = median(lib_us), raw = median(raw_us);
    std::printf("{\"M\": %d, \"N\": %d, \"K\": %d, \"layout\": %d, \"calls\": %d, \"first_call_us\": %.1f, "
                "\"sgemm_tuned_on_us\": %.3f, \"empty_launch_us\": %.3f, \"library_share_us\": %.3f}\n",
                M, N, K, layout, calls, first_us, lib, raw, lib - raw);
    (void)hipFree(A); (void)hipFree(B); (void)hipFree(C);
    return 0;
}
