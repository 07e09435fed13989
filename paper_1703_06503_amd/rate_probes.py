"""Two achievable-rate probes written with the generic tuner (include/kernel_tuner.h), which
double as examples of its use:

    python -m paper_1703_06503_amd.rate_probes

1. What rate can plain v_fma_f32 reach on this device?

A kernel of nothing but independent FMA chains is "tuned" over two parameters: MODE, where the
operands of the FMAs come from (0: three vector registers; 1: the multiplier is a kernel
argument, which the compiler keeps in a scalar register; 2: the same value copied into a vector
register first), and CHAINS, the number of independent chains per thread.  The tuner compiles the
six variants, times each (warm-up, median) and the script turns the times into TFLOP/s.  The
convolution kernels of this library take their filter coefficients as scalar operands (MODE 1);
this probe is where their arithmetic ceiling comes from.

2. What rate can a plain copy reach?  The paper's copy example at the size of the convolution
workloads (one 8192 x 4096 float image read, one written), tuned over floats per thread, vector
width and workgroup size and verified against a scalar reference copy: the practical HBM ceiling
beside which the HBM-bound 3x3 convolution is read."""
import sys

SOURCE = r"""
extern "C" __global__ void fma_loop(const float* in, float* out, int iters,
                                    float s0, float s1, float s2, float s3) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    float acc[CHAINS], x[CHAINS];
    const float a = in[tid & 1023], c = in[(tid + 1) & 1023];
    for (int k = 0; k < CHAINS; ++k) { acc[k] = a + k; x[k] = c * (k + 1); }
#if MODE == 2
    const float v0 = s0 + a * 0.0f, v1 = s1 + a * 0.0f, v2 = s2 + a * 0.0f, v3 = s3 + a * 0.0f;
#endif
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int k = 0; k < CHAINS; ++k) {
#if MODE == 0
                acc[k] = fmaf(acc[k], a, c); acc[k] = fmaf(acc[k], a, c);
                acc[k] = fmaf(acc[k], a, c); acc[k] = fmaf(acc[k], a, c);
#elif MODE == 1
                acc[k] = fmaf(s0, x[k], acc[k]);                 acc[k] = fmaf(s1, x[(k + 1) % CHAINS], acc[k]);
                acc[k] = fmaf(s2, x[(k + 2) % CHAINS], acc[k]);  acc[k] = fmaf(s3, x[(k + 3) % CHAINS], acc[k]);
#else
                acc[k] = fmaf(v0, x[k], acc[k]);                 acc[k] = fmaf(v1, x[(k + 1) % CHAINS], acc[k]);
                acc[k] = fmaf(v2, x[(k + 2) % CHAINS], acc[k]);  acc[k] = fmaf(v3, x[(k + 3) % CHAINS], acc[k]);
#endif
            }
        }
    }
    float s = 0.f;
    for (int k = 0; k < CHAINS; ++k) s += acc[k];
    out[tid] = s;
}
"""
MODES = {0: "three vector registers", 1: "multiplier in a scalar register",
         2: "the same multiplier copied to a vector register"}


COPY = r"""
extern "C" __global__ void copy(const float* in, float* out) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
#if VEC == 4
    const float4* src = reinterpret_cast<const float4*>(in);
    float4* dst = reinterpret_cast<float4*>(out);
    for (int w = 0; w < WPT / 4; ++w) dst[tid * (WPT / 4) + w] = src[tid * (WPT / 4) + w];
#else
    for (int w = 0; w < WPT; ++w) out[tid * WPT + w] = in[tid * WPT + w];
#endif
}
"""
COPY_REF = r"""
extern "C" __global__ void copy_ref(const float* in, float* out) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    out[tid] = in[tid];
}
"""


def copy_rate():
    import numpy as np
    from . import binding as b

    n = 8192 * 4096
    t = b.ktuner_create(COPY, "copy", (n, 1, 1), (1, 1, 1))
    b.ktuner_add_parameter(t, "WPT", [1, 2, 4, 8, 16])
    b.ktuner_add_parameter(t, "VEC", [1, 4])
    b.ktuner_add_parameter(t, "WG", [64, 256, 1024])
    b.ktuner_div_global_size(t, ["WPT", None, None])
    b.ktuner_mul_local_size(t, ["WG", None, None])
    b.ktuner_add_constraint(t, lambda v: v[0] % v[1] == 0, ["WPT", "VEC"])
    b.ktuner_add_argument_input(t, np.random.default_rng(1).standard_normal(n).astype(np.float32))
    b.ktuner_add_argument_output(t, np.zeros(n, np.float32))
    b.ktuner_set_reference(t, COPY_REF, "copy_ref", (n, 1, 1), (256, 1, 1))
    opts = b.tune_opts()
    opts.reps, opts.warmup_ms, opts.cut_factor = 7, 30.0, -1.0
    _, res = b.ktuner_tune(t, b.STRATEGY_FULL, 0, 0, opts)
    print(f"copy of {n} floats: {res.space_size} configurations, {res.failed} failed verification")
    print("| floats per thread | vector width | workgroup | ms | GB/s read + written |")
    print("|---|---|---|---|---|")
    rows = sorted((b.ktuner_time_of(t, i), b.ktuner_space_get(t, i, 3)) for i in range(res.space_size))
    for ms, (wpt, vec, wg) in rows[:5] + rows[-1:]:
        print(f"| {wpt} | {vec} | {wg} | {ms:.4f} | {2 * 4 * n / ms * 1e-6:.0f} |")
    b.ktuner_destroy(t)


def main(argv=None):
    import numpy as np
    from . import binding as b

    iters = 2000
    n = 256 * 4 * 64 * 8                      # eight waves for every SIMD of 256 compute units
    t = b.ktuner_create(SOURCE, "fma_loop", (n, 1, 1), (256, 1, 1))
    b.ktuner_add_parameter(t, "MODE", sorted(MODES))
    b.ktuner_add_parameter(t, "CHAINS", [8, 16])
    b.ktuner_add_argument_input(t, np.random.default_rng(0).uniform(0.5, 1.0, 1024).astype(np.float32))
    b.ktuner_add_argument_output(t, np.zeros(n, np.float32))
    b.ktuner_add_argument_int(t, iters)
    for v in (1e-3, -1e-3, 2e-3, -2e-3):
        b.ktuner_add_argument_float(t, v)
    opts = b.tune_opts()
    opts.reps, opts.warmup_ms, opts.cut_factor = 7, 30.0, -1.0     # time every variant in full
    b.ktuner_tune(t, b.STRATEGY_FULL, 0, 0, opts)
    print("| FMA operands | chains per thread | ms | TFLOP/s |")
    print("|---|---|---|---|")
    for i in range(b.ktuner_space_size(t)):
        mode, chains = b.ktuner_space_get(t, i, 2)
        ms = b.ktuner_time_of(t, i)
        flop = 2.0 * n * iters * 8 * chains    # 2 x 4 FMAs per chain and iteration
        print(f"| {MODES[mode]} | {chains} | {ms:.4f} | {flop / ms * 1e-9:.1f} |")
    b.ktuner_destroy(t)
    print()
    copy_rate()
    return 0


if __name__ == "__main__":
    sys.exit(main())
