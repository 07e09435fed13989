/*
 * conv2d_tuned.h — C ABI of the auto-tuned 2D convolution for AMD MI355X (gfx950): the second
 * kernel family of the library, tuned by the same tuner as the GEMM (same strategies, timing
 * and verification rules; see sgemm_tuned.h, whose status codes, tune_opts and conventions
 * apply here too).
 *
 * The operation is the one of the CLTune paper's section "Case-study: 2D convolution":
 *
 *     B[y][x] = w * sum_{j < Yf} sum_{i < Xf} F[j][i] * A[y + j][x + i]      0 <= x < X, 0 <= y < Y
 *
 * (the paper's sum with its indices shifted to start at zero; the filter is not flipped).
 *   A  DEVICE, the input image stored WITH its halo: Y + Yf - 1 rows of at least X + Xf - 1
 *      floats, leading dimension lda >= X + Xf - 1, x fastest.  The caller provides the halo
 *      values (zeros, mirrored pixels, ...): the paper leaves the image border open.
 *   F  DEVICE, the filter, Yf rows of Xf floats, contiguous.
 *   B  DEVICE, the output, Y rows of X floats, leading dimension ldb >= X.  Must not overlap A.
 *   1 <= Xf, Yf <= 31.  X == 0 or Y == 0: no-op.
 * Filter sizes are compile-time constants of the generated kernels, as in the paper; every
 * (configuration, Xf, Yf) is its own variant in the kernel cache.
 */
#ifndef CONV2D_TUNED_H
#define CONV2D_TUNED_H

#include "sgemm_tuned.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One configuration of the kernel family (section "Tuning parameters" of the convolution case
 * study; table "Best-found parameters for 2D convolution" for the value lists). */
typedef struct conv2d_config {
    int xwg, ywg;   /* computing threads of a workgroup: {8,16,32,64} each                  */
    int xwpt, ywpt; /* outputs per thread in x and y: {1,2,4,8} each                        */
    int lmem;       /* the paper's L$: 0 = caches only, 1 = input tile in LDS, loaded by the
                       computing threads together, 2 = loaded by one thread per rectangle
                       with helper threads for the halo                                     */
    int vw;         /* vector width of the stores (and of the loads with lmem = 2): divides
                       xwpt; used only where lda, ldb and the pointers are aligned for it   */
    int pad;        /* extra floats per LDS row: {0,1}; 0 when lmem = 0                      */
    int unr;        /* 1 = loops over the filter unrolled, 0 = kept as loops                 */
} conv2d_config;

#define CONV2D_MAX_FILTER 31

/* ---- the space [host] ------------------------------------------------------------------
 * Valid configurations for an Xf x Yf filter, in lexicographic order (xwg slowest).  The
 * constraints: vw divides xwpt; pad = 0 when lmem = 0; at most 1024 threads per workgroup,
 * helper threads included; the LDS tile fits 160 KiB. */
int conv2d_space_size(int Xf, int Yf);
int conv2d_space_get(int Xf, int Yf, int index, conv2d_config *out);
int conv2d_space_find(int Xf, int Yf, const conv2d_config *cfg);   /* index or SGEMM_E_INVALID */
int conv2d_config_check(const conv2d_config *cfg, int Xf, int Yf); /* SGEMM_OK or _E_INVALID   */
int conv2d_config_lds_bytes(const conv2d_config *cfg, int Xf, int Yf);
int conv2d_config_threads(const conv2d_config *cfg, int Xf, int Yf);

/* Compiles (or finds in the kernel cache) the variant; needs no GPU.  edge = 1: the build
 * for X or Y that are not multiples of the workgroup's tile; vector = 0: the build with
 * scalar loads and stores that misaligned operands get.  info may be null. */
int conv2d_kernel_compile(const conv2d_config *cfg, int Xf, int Yf, int edge, int vector,
                          sgemm_kernel_info *info);

/* ---- running ---------------------------------------------------------------------------
 * One convolution with the given configuration on the given HIP stream (null = default).
 * 0 <= X, Y <= 2^31 - 1025 and at most 65535 rows of workgroups (Y <= 65535 * YWG * YWPT), else
 * SGEMM_E_BADARG. */
int conv2d_run_config(void *hip_stream, const conv2d_config *cfg, int X, int Y, int Xf, int Yf,
                      float w, const float *F, const float *A, int lda, float *B, int ldb);

/* The reference kernel every tuned variant is compared with (one thread per output). */
int conv2d_reference(void *hip_stream, int X, int Y, int Xf, int Yf, float w, const float *F,
                     const float *A, int lda, float *B, int ldb);

/* With the best configuration known for (X, Y, Xf, Yf): the one a conv2d_tune() of this process
 * or conv2d_config_set() stored; else that of the nearest image size with the same filter; else
 * a built-in default (the winner of a recorded full search with a 3 x 3, 7 x 7 or 11 x 11
 * filter, whichever is nearest in number of taps; a configuration with the filter loops kept as
 * loops for filters of more than 121 taps).  Never tunes.  Uses the
 * stream of sgemm_set_stream(). */
int conv2d_tuned(int X, int Y, int Xf, int Yf, float w, const float *F, const float *A, int lda,
                 float *B, int ldb);
int conv2d_config_set(int X, int Y, int Xf, int Yf, const conv2d_config *cfg, float ms);
int conv2d_config_select(int X, int Y, int Xf, int Yf, conv2d_config *out); /* 1 = exact, 0 = else */

/* [host] The table of best configurations as a text file, one line per problem
 * ("X Y Xf Yf ms XWG YWG XWPT YWPT LMEM VW PAD UNR"; '#' starts a comment).  save returns the
 * number of entries written; load merges (a faster or first entry wins; lines this build cannot
 * run are skipped) and returns the number of lines taken; clear empties the table. */
int conv2d_cache_save(const char *path);
int conv2d_cache_load(const char *path);
int conv2d_cache_clear(void);

/* ---- tuning ----------------------------------------------------------------------------
 * Searches the space of an Xf x Yf filter on an X x Y image with library-owned seeded operands
 * (image rows padded to a multiple of 16 floats, so that no vector width is ruled out by
 * alignment), exactly as tune_ex() does for the GEMM: every configuration is compiled, run once and
 * compared with the reference kernel under
 *     |B - B_ref| <= 1e-5 * Xf * Yf * |w| * max|F| * max|A| + 1e-6 * |B_ref|,
 * then warmed up and timed (median).  strategy, budget, seed and the fields warmup, reps,
 * verify_off, cut_factor, warmup_ms, sa_T, sa_raw_ms, pso_*, random_fraction, log_path and
 * warm_start (negative form) of opts mean what they mean there; the other fields are ignored.
 * Returns the number of configurations evaluated, or a negative status; the best is stored for
 * conv2d_tuned(). */
typedef struct conv2d_tune_result {
    conv2d_config best;
    float best_ms;
    float best_gflops;  /* (1 + 2 Xf Yf) X Y / time, the paper's count                        */
    float best_gbs;     /* 2 X Y floats / time, the paper's count of the image traffic        */
    int best_index, evaluations, failed, space_size, evals_to_best;
    float total_ms, compile_ms;
    int reserved[4];
} conv2d_tune_result;

int conv2d_tune(int X, int Y, int Xf, int Yf, float w, int strategy, int budget,
                unsigned long long seed, const tune_opts *opts, conv2d_tune_result *out);

/* The same strategies on a recorded table: ms_table[i] = milliseconds of configuration i of the
 * (Xf, Yf) space, <= 0 or non-finite = failed; visited (may be null) receives up to visited_cap
 * configuration indices in evaluation order.  [host] */
int conv2d_tune_replay(int Xf, int Yf, const float *ms_table, int table_len, int strategy,
                       int budget, unsigned long long seed, const tune_opts *opts, int *visited,
                       int visited_cap, conv2d_tune_result *out);

#ifdef __cplusplus
}
#endif
#endif
