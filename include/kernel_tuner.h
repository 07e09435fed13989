/*
 * kernel_tuner.h — C ABI of the generic tuner: the auto-tuning method of the CLTune paper
 * (section "CLTune: an auto-tuner for OpenCL kernels" and its "Advanced usage") for ANY HIP
 * kernel on AMD MI355X (gfx950), not only the two kernel families the library ships.
 *
 * The caller hands over the kernel's source text, names integer tuning parameters with their
 * value lists, says how the thread counts follow from the parameters, optionally adds
 * constraints and a reference kernel, and lists the kernel's arguments.  The tuner builds the
 * constraint-pruned space, compiles each configuration with the parameters as -DNAME=value
 * macros (same kernel cache as the rest of the library), runs it on a fresh device copy of the
 * arguments, compares every output argument with the reference kernel's, times it (warm-up and
 * median, as tune_ex() does) and searches with the four strategies of sgemm_tuned.h.
 *
 * Conventions: extern "C"; int status returns (SGEMM_OK or negative SGEMM_E_* of sgemm_tuned.h;
 * sgemm_last_error() has the detail); all pointers are HOST memory owned by the caller -- the
 * tuner allocates, fills and frees the device buffers itself, so that, as in the paper, the
 * caller never touches the device API.  A tuner handle is not thread-safe.
 * The kernel must be declared extern "C" __global__ in the source; its parameters are the
 * arguments in the order they were added.
 */
#ifndef KERNEL_TUNER_H
#define KERNEL_TUNER_H

#include <stddef.h>

#include "sgemm_tuned.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ktuner ktuner; /* opaque */

#define KTUNER_MAX_PARAMETERS 15

/* A tuner for kernel `entry` of `source` (HIP source text, copied).  global[d] = total number of
 * threads in dimension d and local[d] = threads of a workgroup in dimension d (both for
 * d = 0, 1, 2; use 1 for unused dimensions) BEFORE the modifiers below are applied -- the
 * paper's global and local sizes.  Returns NULL on bad arguments. */
ktuner *ktuner_create(const char *source, const char *entry, const int global[3], const int local[3]);
void ktuner_destroy(ktuner *t);

/* A tuning parameter: reaches the kernel as the macro NAME with one of the n values.  At most
 * KTUNER_MAX_PARAMETERS; names must be distinct C identifiers. */
int ktuner_add_parameter(ktuner *t, const char *name, const int *values, int n);

/* Thread-count modifiers ("Advanced usage"): multiply or divide the global or local size of
 * dimension d by the value of parameter names[d]; names[d] == NULL leaves dimension d alone.
 * Several modifiers apply in the order they were added.  A configuration whose sizes do not
 * divide, whose global size is not a multiple of its local size, or whose workgroup has more
 * than 1024 threads is not part of the space (the device limits the paper imposes itself). */
int ktuner_mul_global_size(ktuner *t, const char *const names[3]);
int ktuner_div_global_size(ktuner *t, const char *const names[3]);
int ktuner_mul_local_size(ktuner *t, const char *const names[3]);
int ktuner_div_local_size(ktuner *t, const char *const names[3]);

/* A constraint on the n named parameters: fn(values, user) is called with their values in the
 * order of `names` and returns non-zero for an allowed combination. */
typedef int (*ktuner_constraint_fn)(const int *values, void *user);
int ktuner_add_constraint(ktuner *t, ktuner_constraint_fn fn, const char *const *names, int n, void *user);

/* The kernel's arguments, in order.  Buffers are `bytes` of HOST data copied to the device once;
 * before every configuration is run, each device buffer is restored from that copy ("a fresh
 * device-copy of the supplied arguments").  Output buffers are float arrays (bytes a multiple
 * of 4) that are compared with the reference kernel's after the run. */
int ktuner_add_argument_input(ktuner *t, const void *host, size_t bytes);
int ktuner_add_argument_output(ktuner *t, const void *host_initial, size_t bytes);
int ktuner_add_argument_int(ktuner *t, int value);
int ktuner_add_argument_float(ktuner *t, float value);

/* The reference kernel: same arguments, fixed thread counts, no parameters.  Without one,
 * configurations are timed but not verified.  Outputs match when
 * |out - ref| <= abs_tol + rel_tol * |ref| (defaults 1e-6 * max|ref| and 1e-5; set either
 * negative to keep its default). */
int ktuner_set_reference(ktuner *t, const char *source, const char *entry, const int global[3],
                         const int local[3]);
int ktuner_set_tolerance(ktuner *t, float abs_tol, float rel_tol);

/* [host] The space: valid configurations in lexicographic order (first parameter slowest);
 * values receives one value per parameter, in the order the parameters were added. */
int ktuner_space_size(ktuner *t);
int ktuner_space_get(ktuner *t, int index, int *values);
/* [host] Compiles configuration `index` (or finds it in the kernel cache); info may be null. */
int ktuner_compile(ktuner *t, int index, sgemm_kernel_info *info);
/* [host] Grid and workgroup of configuration `index`: grid[d] workgroups of block[d] threads. */
int ktuner_launch_shape(ktuner *t, int index, int grid[3], int block[3]);

/* Runs the search on the current device.  strategy, budget, seed and the fields warmup, reps,
 * verify_off, cut_factor, warmup_ms, sa_T, sa_raw_ms, pso_*, random_fraction, log_path and
 * warm_start (negative form) of opts are those of tune_ex().  Returns the number of
 * configurations evaluated or a negative status. */
typedef struct ktuner_result {
    int best_index;      /* -1 when every configuration failed                             */
    float best_ms;
    int evaluations, failed, space_size, evals_to_best;
    int failed_verify;   /* of the failed: output differed from the reference kernel's      */
    float total_ms, compile_ms;
    int reserved[7];
} ktuner_result;
int ktuner_tune(ktuner *t, int strategy, int budget, unsigned long long seed, const tune_opts *opts,
                ktuner_result *out);

/* After ktuner_tune(): milliseconds of configuration `index` (0 if it was not evaluated,
 * negative if it failed), and a copy of output argument `which` (0-based among the outputs) as
 * the best configuration left it, for callers that want to inspect the result. */
float ktuner_time_of(ktuner *t, int index);
int ktuner_read_output(ktuner *t, int which, void *host, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif
