// Small fixed kernels of the tuning harness (compiled ahead of time for gfx950): the
// reference GEMM that every tuned variant is verified against, operand fill, the tolerance
// check, |x| maximum, and the C = beta*C scaling used when alpha == 0 or K == 0.
#include <hip/hip_runtime.h>

#include <mutex>

#include "util_kernels.h"

namespace {

// One thread per element of C; products and sums in double in increasing k.  This is the
// "reference kernel" of the paper's result verification (section "Advanced usage").
__global__ void reference_kernel(int M, int N, int K, float alpha, const float *__restrict__ A,
                                 int lda, const float *__restrict__ B, int ldb, float beta,
                                 float *__restrict__ C, int ldc, int layout) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    // rows are strided over the grid: the host caps the number of workgroup rows
    for (long long i = (long long)blockIdx.y * blockDim.y + threadIdx.y; i < M; i += (long long)gridDim.y * blockDim.y) {
        double sum = 0.0;
        if (alpha != 0.0f) {
            for (int k = 0; k < K; ++k) {
                const float a = (layout & 1) ? A[(size_t)k * lda + i] : A[(size_t)i * lda + k];
                const float b = (layout & 2) ? B[(size_t)j * ldb + k] : B[(size_t)k * ldb + j];
                sum += (double)a * (double)b;
            }
        }
        double r = (double)alpha * sum;
        float *p = C + (size_t)i * ldc + j;
        if (beta != 0.0f) r += (double)beta * (double)*p;
        *p = (float)r;
    }
}

__global__ void scale_kernel(int M, int N, float beta, float *__restrict__ C, int ldc) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    for (long long i = (long long)blockIdx.y * blockDim.y + threadIdx.y; i < M; i += (long long)gridDim.y * blockDim.y) {
        float *p = C + (size_t)i * ldc + j;
        *p = (beta == 0.0f) ? 0.0f : beta * *p;
    }
}

__device__ inline unsigned long long mix64(unsigned long long z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// rows x cols matrix with leading dimension ld, i.i.d. uniform on [-1, 1): a function of
// (seed, row, col) only, so the values do not depend on ld or on the launch shape.
__global__ void fill_uniform_kernel(float *__restrict__ dst, int rows, int cols, int ld,
                                    unsigned long long seed) {
    const size_t n = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / cols, c = e % cols;
        const unsigned long long u = mix64(seed ^ mix64(e));
        dst[r * ld + c] = (float)((double)(u >> 11) * (2.0 / 9007199254740992.0) - 1.0);
    }
}

// out[0] = max |x| over a rows x cols matrix, as float bits (non-negative floats order like
// their bit patterns).  *out must be zeroed by the caller.
__global__ void absmax_kernel(const float *__restrict__ src, int rows, int cols, int ld,
                              unsigned int *out) {
    const size_t n = (size_t)rows * cols;
    float m = 0.0f;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x) {
        const float v = fabsf(src[(e / cols) * ld + e % cols]);
        if (v > m || v != v) m = (v != v) ? __uint_as_float(0x7f800000u) : v;
    }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((threadIdx.x & 63) == 0) atomicMax(out, __float_as_uint(m));
}

// Counts elements with |got - ref| > abs_tol + rel_tol*|ref| (NaN in exactly one of the two
// counts as a violation) and keeps the largest excess ratio err / bound.
__global__ void compare_kernel(const float *__restrict__ got, int ldg,
                               const float *__restrict__ ref, int ldr, int M, int N,
                               float abs_tol, float rel_tol, unsigned int *violations,
                               unsigned int *worst_ratio_bits) {
    const size_t n = (size_t)M * N;
    unsigned int bad = 0;
    float worst = 0.0f;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x) {
        const float g = got[(e / N) * ldg + e % N];
        const float r = ref[(e / N) * ldr + e % N];
        const bool gn = (g != g), rn = (r != r);
        if (gn || rn) {
            if (gn != rn) { ++bad; worst = __uint_as_float(0x7f800000u); }
            continue;
        }
        if (g == r) continue; // also covers equal infinities
        const float bound = abs_tol + rel_tol * fabsf(r);
        const float err = fabsf(g - r);
        if (!(err <= bound)) ++bad;
        const float ratio = bound > 0.0f ? err / bound : __uint_as_float(0x7f800000u);
        if (ratio > worst) worst = ratio;
    }
    for (int o = 32; o > 0; o >>= 1) {
        bad += __shfl_xor(bad, o);
        worst = fmaxf(worst, __shfl_xor(worst, o));
    }
    if ((threadIdx.x & 63) == 0) {
        if (bad) atomicAdd(violations, bad);
        atomicMax(worst_ratio_bits, __float_as_uint(worst));
    }
}

__global__ void copy2d_kernel(float *__restrict__ dst, int ldd, const float *__restrict__ src,
                              int lds_, int rows, int cols) {
    const size_t n = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x)
        dst[(e / cols) * ldd + e % cols] = src[(e / cols) * lds_ + e % cols];
}

// C = alpha * (P[0] + P[1] + ... + P[planes-1]) + beta * C, planes added in index order so the
// result does not depend on the launch; P[s] is an M x N matrix (leading dimension N) at
// P + s * plane.  VW floats per thread (4 when N, ldc and both pointers allow 16-byte access).
template <int VW> struct reduce_vec;
template <> struct reduce_vec<1> { typedef float type; };
template <> struct reduce_vec<4> { typedef float type __attribute__((ext_vector_type(4))); };

// The planes are added in index order (so the result does not depend on timing), but their
// loads are independent: four at a time are requested before the first of them is added, so an
// element waits for memory once per four planes instead of once per plane.  The old C, when it
// is needed, is requested with the first group.
template <int VW>
__global__ void splitk_reduce_kernel(int M, int N, int planes, const float *__restrict__ P,
                                     size_t plane, float alpha, float beta, float *__restrict__ C,
                                     int ldc) {
    typedef typename reduce_vec<VW>::type vec;
    const int nv = N / VW;
    const size_t n = (size_t)M * nv;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x) {
        size_t r, c;
        if (n <= 0xffffffffu) { // the usual case: 32-bit division
            r = (unsigned)e / (unsigned)nv;
            c = (size_t)((unsigned)e % (unsigned)nv) * VW;
        } else {
            r = e / nv;
            c = (e % nv) * VW;
        }
        const float *p = P + r * (size_t)N + c;
        vec *out = reinterpret_cast<vec *>(C + r * (size_t)ldc + c);
        vec old = {};
        if (beta != 0.0f) old = *out; // C is read only when beta != 0
#define PLANE(i) (*reinterpret_cast<const vec *>(p + (size_t)(i) * plane))
        vec acc;
        int s;
        if (planes >= 8) {
            const vec v0 = PLANE(0), v1 = PLANE(1), v2 = PLANE(2), v3 = PLANE(3), v4 = PLANE(4), v5 = PLANE(5),
                      v6 = PLANE(6), v7 = PLANE(7);
            acc = v0; acc += v1; acc += v2; acc += v3; acc += v4; acc += v5; acc += v6; acc += v7;
            s = 8;
        } else if (planes >= 4) {
            const vec v0 = PLANE(0), v1 = PLANE(1), v2 = PLANE(2), v3 = PLANE(3);
            acc = v0; acc += v1; acc += v2; acc += v3;
            s = 4;
        } else {
            acc = PLANE(0);
            s = 1;
        }
        for (; s + 4 <= planes; s += 4) {
            const vec v0 = PLANE(s), v1 = PLANE(s + 1), v2 = PLANE(s + 2), v3 = PLANE(s + 3);
            acc += v0; acc += v1; acc += v2; acc += v3;
        }
        if (s + 2 <= planes) {
            const vec v0 = PLANE(s), v1 = PLANE(s + 1);
            acc += v0; acc += v1;
            s += 2;
        }
        if (s < planes) acc += PLANE(s);
#undef PLANE
        acc = alpha * acc;
        if (beta != 0.0f) acc += beta * old;
        *out = acc;
    }
}

// dst (rows_d x cols_d, leading dimension ldd) = src (rows_s x cols_s, leading dimension lds_)
// in its top-left corner, zeros elsewhere: the padding that lets an unguarded GEMM variant
// run on a problem that is not a multiple of its tile (the paper's pre-processing kernel).
__global__ void pad_copy_kernel(float *__restrict__ dst, int ldd, int rows_d, int cols_d,
                                const float *__restrict__ src, int lds_, int rows_s, int cols_s) {
    const size_t n = (size_t)rows_d * cols_d;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / cols_d, c = e % cols_d;
        dst[r * ldd + c] = (r < (size_t)rows_s && c < (size_t)cols_s) ? src[r * lds_ + c] : 0.0f;
    }
}

// The convolution every tuned variant is compared with: one thread per output, taps added in
// the order j outer, i inner (paper: "Case-study: 2D convolution", the equation for B[x,y]).
__global__ void conv2d_reference_kernel(int X, int Y, int Xf, int Yf, float w,
                                        const float *__restrict__ F, const float *__restrict__ A,
                                        int lda, float *__restrict__ B, int ldb) {
    const int x = blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= X) return;
    for (long long y = (long long)blockIdx.y * blockDim.y + threadIdx.y; y < Y; y += (long long)gridDim.y * blockDim.y) {
        float acc = 0.0f;
        for (int j = 0; j < Yf; ++j)
            for (int i = 0; i < Xf; ++i) acc = fmaf(F[j * Xf + i], A[(size_t)(y + j) * lda + x + i], acc);
        B[(size_t)y * ldb + x] = w * acc;
    }
}

// Every element of an M x N matrix (leading dimension ld) gets the same bit pattern: the
// sentinel (a NaN) that an output holds before a configuration's verified run, so that an
// element the variant fails to write cannot pass for the previous variant's correct value.
__global__ void fill_bits_kernel(float *__restrict__ dst, int rows, int cols, int ld, unsigned int bits) {
    const size_t n = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
         e += (size_t)gridDim.x * blockDim.x)
        dst[(e / cols) * ld + e % cols] = __uint_as_float(bits);
}

__global__ void zero_u32_kernel(unsigned int *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Device memory that exists without any allocation call: the split-K planes of
// sgemm_tuned_noalloc().  One copy per GPU, held until the process ends.  Host code never uses
// this name as an address; it asks the runtime for the array's device address (below).
static __device__ __align__(256) float scratch[sgemm_util::kScratchFloats];

// The second grid dimension holds at most 65535 workgroups: kernels that put matrix rows there
// stride over them.
inline unsigned rows_of_workgroups(int rows, int per_workgroup) {
    const long long g = ((long long)rows + per_workgroup - 1) / per_workgroup;
    return (unsigned)(g > 65535 ? 65535 : g);
}

inline int grid_for(size_t n, int block) {
    size_t g = (n + block - 1) / block;
    if (g > 256 * 16) g = 256 * 16;
    if (g < 1) g = 1;
    return (int)g;
}

} // namespace

namespace sgemm_util {

hipError_t launch_reference(hipStream_t s, int M, int N, int K, float alpha, const float *A,
                            int lda, const float *B, int ldb, float beta, float *C, int ldc,
                            int layout) {
    if (M == 0 || N == 0) return hipSuccess;
    dim3 block(64, 4), grid((N + 63) / 64, rows_of_workgroups(M, 4));
    hipLaunchKernelGGL(reference_kernel, grid, block, 0, s, M, N, K, alpha, A, lda, B, ldb, beta,
                       C, ldc, layout);
    return hipGetLastError();
}

hipError_t launch_scale(hipStream_t s, int M, int N, float beta, float *C, int ldc) {
    if (M == 0 || N == 0) return hipSuccess;
    dim3 block(64, 4), grid((N + 63) / 64, rows_of_workgroups(M, 4));
    hipLaunchKernelGGL(scale_kernel, grid, block, 0, s, M, N, beta, C, ldc);
    return hipGetLastError();
}

hipError_t launch_fill_uniform(hipStream_t s, float *dst, int rows, int cols, int ld,
                               unsigned long long seed) {
    const size_t n = (size_t)rows * cols;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_uniform_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, rows,
                       cols, ld, seed);
    return hipGetLastError();
}

hipError_t launch_absmax(hipStream_t s, const float *src, int rows, int cols, int ld,
                         unsigned int *out_bits) {
    hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, s, out_bits, 1);
    const size_t n = (size_t)rows * cols;
    if (n == 0) return hipGetLastError();
    hipLaunchKernelGGL(absmax_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, src, rows, cols, ld,
                       out_bits);
    return hipGetLastError();
}

hipError_t launch_compare(hipStream_t s, const float *got, int ldg, const float *ref, int ldr,
                          int M, int N, float abs_tol, float rel_tol, unsigned int *two_words) {
    hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, s, two_words, 2);
    const size_t n = (size_t)M * N;
    if (n == 0) return hipGetLastError();
    hipLaunchKernelGGL(compare_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, got, ldg, ref, ldr,
                       M, N, abs_tol, rel_tol, two_words, two_words + 1);
    return hipGetLastError();
}

hipError_t launch_splitk_reduce(hipStream_t s, int M, int N, int planes, const float *P,
                                size_t plane, float alpha, float beta, float *C, int ldc) {
    if (M == 0 || N == 0 || planes <= 0) return hipSuccess;
    const bool wide = N % 4 == 0 && ldc % 4 == 0 && plane % 4 == 0 &&
                      (reinterpret_cast<uintptr_t>(P) % 16) == 0 &&
                      (reinterpret_cast<uintptr_t>(C) % 16) == 0;
    if (wide) {
        const size_t n = (size_t)M * (N / 4);
        hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3(grid_for(n, 256)), dim3(256), 0, s, M, N,
                           planes, P, plane, alpha, beta, C, ldc);
    } else {
        const size_t n = (size_t)M * N;
        hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3(grid_for(n, 256)), dim3(256), 0, s, M, N,
                           planes, P, plane, alpha, beta, C, ldc);
    }
    return hipGetLastError();
}

hipError_t launch_fill_bits(hipStream_t s, float *dst, int rows, int cols, int ld, unsigned int bits) {
    const size_t n = (size_t)rows * cols;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_bits_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, rows, cols, ld, bits);
    return hipGetLastError();
}

hipError_t scratch_of_current_device(float **ptr) {
    static std::mutex mu;
    static float *known[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!known[dev]) {
        // each GPU holds its own copy of the array at its own address
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        known[dev] = static_cast<float *>(p);
    }
    *ptr = known[dev];
    return hipSuccess;
}

hipError_t launch_conv2d_reference(hipStream_t s, int X, int Y, int Xf, int Yf, float w, const float *F,
                                   const float *A, int lda, float *B, int ldb) {
    if (X <= 0 || Y <= 0) return hipSuccess;
    const dim3 block(64, 4);
    hipLaunchKernelGGL(conv2d_reference_kernel, dim3((X + 63) / 64, rows_of_workgroups(Y, 4)), block, 0, s, X, Y,
                       Xf, Yf, w, F, A, lda, B, ldb);
    return hipGetLastError();
}

hipError_t launch_pad_copy(hipStream_t s, float *dst, int ldd, int rows_d, int cols_d,
                           const float *src, int lds_, int rows_s, int cols_s) {
    const size_t n = (size_t)rows_d * cols_d;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(pad_copy_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, ldd, rows_d,
                       cols_d, src, lds_, rows_s, cols_s);
    return hipGetLastError();
}

hipError_t launch_copy2d(hipStream_t s, float *dst, int ldd, const float *src, int lds_, int rows,
                         int cols) {
    const size_t n = (size_t)rows * cols;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(copy2d_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, ldd, src, lds_,
                       rows, cols);
    return hipGetLastError();
}

} // namespace sgemm_util
