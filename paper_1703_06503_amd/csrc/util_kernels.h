// Host-callable launchers of the harness's fixed kernels (util_kernels.hip).
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

namespace sgemm_util {

hipError_t launch_reference(hipStream_t s, int M, int N, int K, float alpha, const float *A,
                            int lda, const float *B, int ldb, float beta, float *C, int ldc,
                            int layout);
hipError_t launch_scale(hipStream_t s, int M, int N, float beta, float *C, int ldc);
hipError_t launch_fill_uniform(hipStream_t s, float *dst, int rows, int cols, int ld,
                               unsigned long long seed);
// *out_bits (device) receives the bit pattern of max |x|.
hipError_t launch_absmax(hipStream_t s, const float *src, int rows, int cols, int ld,
                         unsigned int *out_bits);
// two_words (device): [0] = number of elements outside abs_tol + rel_tol*|ref|,
// [1] = bit pattern of the largest err / bound.
hipError_t launch_compare(hipStream_t s, const float *got, int ldg, const float *ref, int ldr,
                          int M, int N, float abs_tol, float rel_tol, unsigned int *two_words);
// C = alpha * (P[0] + ... + P[planes-1]) + beta * C; P[s] = M x N floats (ld N) at P + s*plane.
hipError_t launch_splitk_reduce(hipStream_t s, int M, int N, int planes, const float *P,
                                size_t plane, float alpha, float beta, float *C, int ldc);
// B[y][x] = w * sum_j sum_i F[j][i] * A[y+j][x+i]; A holds the halo.
hipError_t launch_conv2d_reference(hipStream_t s, int X, int Y, int Xf, int Yf, float w, const float *F,
                                   const float *A, int lda, float *B, int ldb);
// dst (rows_d x cols_d) = src (rows_s x cols_s) in the top-left corner, zeros elsewhere.
hipError_t launch_pad_copy(hipStream_t s, float *dst, int ldd, int rows_d, int cols_d,
                           const float *src, int lds_, int rows_s, int cols_s);
// Every element of a rows x cols matrix = the float with this bit pattern.
hipError_t launch_fill_bits(hipStream_t s, float *dst, int rows, int cols, int ld, unsigned int bits);

// The library's statically allocated device scratch memory (kScratchFloats floats, 256-byte
// aligned, one copy per GPU, contents kept between calls): *ptr receives its address on the
// current device.  The first call on a device looks the address up; no call allocates.
constexpr size_t kScratchFloats = (size_t)8 << 20; // 32 MiB
constexpr int kMaxDevices = 64;
hipError_t scratch_of_current_device(float **ptr);

hipError_t launch_copy2d(hipStream_t s, float *dst, int ldd, const float *src, int lds_, int rows,
                         int cols);

} // namespace sgemm_util
