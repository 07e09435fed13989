"""What rate can plain v_fma_f32 reach on this device?  A probe written with the generic tuner
(include/kernel_tuner.h), and an example of its use:

    python -m paper_1703_06503_amd.fma_probe

A kernel of nothing but independent FMA chains is "tuned" over two parameters: MODE, where the
operands of the FMAs come from (0: three vector registers; 1: the multiplier is a kernel
argument, which the compiler keeps in a scalar register; 2: the same value copied into a vector
register first), and CHAINS, the number of independent chains per thread.  The tuner compiles the
six variants, times each (warm-up, median) and the script turns the times into TFLOP/s.  The
convolution kernels of this library take their filter coefficients as scalar operands (MODE 1);
this probe is where their arithmetic ceiling comes from."""
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
    return 0


if __name__ == "__main__":
    sys.exit(main())
