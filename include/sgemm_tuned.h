/*
 * sgemm_tuned.h — C ABI of the auto-tuned single-precision GEMM for AMD MI355X (gfx950).
 *
 * The library holds a family of GEMM kernels generated from one HIP source by compile-time
 * parameters, the tuner that searches that parameter space (full, random, simulated
 * annealing, particle swarm), and a per-shape cache of the best configuration found.
 * It follows the auto-tuning method of the CLTune paper (sections "CLTune: an auto-tuner
 * for OpenCL kernels" and "Case-study: matrix-multiplication"), redesigned for gfx950.
 *
 * Conventions for every entry point
 *   - All functions are extern "C", never throw, and return an int status: SGEMM_OK (0) or
 *     a negative SGEMM_E_* code (sgemm_status_string() names it).  Functions documented as
 *     returning a count return a value >= 0 on success.
 *   - A, B, C are DEVICE pointers (for example torch.Tensor.data_ptr() on a ROCm tensor).
 *     The caller owns them; the library never frees or keeps them.
 *   - Everything else (config structs, tables, strings, result structs) is HOST memory
 *     owned by the caller.
 *   - Launches are asynchronous on the given HIP stream; an error detected by the launch
 *     call is returned, a later device fault is not.
 *   - Functions marked [host] need no GPU and touch no GPU state.
 */
#ifndef SGEMM_TUNED_H
#define SGEMM_TUNED_H

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---------------------------------------------------------------- */
#define SGEMM_OK 0
#define SGEMM_E_BADARG (-1)   /* negative size, leading dimension too small (or lda / ldb
                                 above SGEMM_MAX_LEADING_DIM), null pointer for a non-empty
                                 operand, unknown layout/strategy/preset */
#define SGEMM_E_NOCONFIG (-2) /* the search space holds no valid configuration */
#define SGEMM_E_COMPILE (-3)  /* the kernel generator failed to compile a variant */
#define SGEMM_E_LAUNCH (-4)   /* HIP refused a module load, launch, allocation or copy */
#define SGEMM_E_VERIFY (-5)   /* a variant's output disagreed with the reference kernel */
#define SGEMM_E_INVALID (-6)  /* configuration violates a constraint of the kernel family */
#define SGEMM_E_IO (-7)       /* cache file could not be read or written */
#define SGEMM_E_NODEVICE (-8) /* no usable HIP device */
#define SGEMM_E_RESOURCE (-9) /* variant compiled but spills registers or exceeds LDS; or a call
                                 that may not allocate needs more scratch memory than exists */
#define SGEMM_E_NOTREADY (-10) /* sgemm_tuned_noalloc(): this call's variant is not loaded yet */

/* ---- layout bits ------------------------------------------------------------------
 * The paper's kernel multiplies A^T by B, i.e. it expects A stored K x M.  Here that
 * storage is selected per call: bit 0 set = A stored K x M (row-major, lda >= M), clear =
 * A stored M x K (lda >= K); bit 1 set = B stored N x K (ldb >= K), clear = B stored K x N
 * (ldb >= N).  C is always M x N row-major (ldc >= N).  Leading dimensions in elements;
 * lda and ldb at most SGEMM_MAX_LEADING_DIM (a tile of A or B must lie within the 2 GiB that
 * the kernels address with 32-bit offsets from the tile's origin). */
#define SGEMM_MAX_LEADING_DIM (1 << 20)
#define SGEMM_LAYOUT_A_TRANSPOSED 1
#define SGEMM_LAYOUT_B_TRANSPOSED 2

/* ---- search strategies (section "Search strategies and search-space properties") ---- */
#define SGEMM_STRATEGY_FULL 0
#define SGEMM_STRATEGY_RANDOM 1
#define SGEMM_STRATEGY_ANNEALING 2
#define SGEMM_STRATEGY_PSO 3

/* ---- search-space presets ---------------------------------------------------------- */
#define SGEMM_SPACE_FULL 0  /* the full gfx950 space (about 10^4 valid configurations) */
#define SGEMM_SPACE_SMALL 1 /* 16 configurations: MWG,NWG in {32,64}, KWG in {8,16},
                               LDS staging on/off; everything else fixed */
#define SGEMM_SPACE_MFMA 2  /* matrix-core variants only, both operands staged, wider value
                               lists (workgroups up to 512 threads, both MFMA shapes) */
#define SGEMM_SPACE_DIRECT 4 /* matrix-core variants whose tiles reach LDS by LDS-direct loads
                               (sa = sb = 2), with 2 to 4 LDS buffers per tile (ns), the tile
                               edges and split-K values of SGEMM_SPACE_EXT */
#define SGEMM_SPACE_EXT 3   /* SGEMM_SPACE_MFMA plus tile edges 96 and 192, K slabs of 64 and
                               split K (sk up to 16): for sizes that powers of two tile badly
                               and for shapes with few tiles and a long K */

#define SGEMM_SPACE_KSPLIT 6 /* matrix-core variants with small tiles (32 to 128) whose waves share
                               out the K slab (ksw 2 or 4), with split K 1, 2, 4: for problems too
                               small to fill the chip with large tiles */
#define SGEMM_SPACE_CUSTOM 5 /* value lists given by the caller: sgemm_space_define_custom() */

/* One point of the parameter space.  Names follow the paper's GEMM parameters (list in
 * "Tuning parameters" of the matrix-multiplication case study): the workgroup tile
 * Mwg/Nwg/Kwg, the workgroup shape MdimC x NdimC (so each thread owns Mwi = Mwg/MdimC by
 * Nwi = Nwg/NdimC accumulators), the vector widths of the off-chip loads, local-memory
 * staging per operand, and the unroll factor Kwi of the Kwg loop.  `pad`, `mfma`, `grp`,
 * `sk`, `ns` and `ksw` are gfx950 additions.  All fields are plain ints so the struct is an int[16]. */
typedef struct sgemm_config {
    int mwg, nwg, kwg; /* workgroup macro-tile of C (mwg x nwg: each 2^a, 3*2^a, 5*2^a or 7*2^a) and K slab
                          per step (power of two)                                          */
    int mdimc, ndimc;  /* threads per workgroup = mdimc * ndimc (multiple of 64), times ksw */
    int vwm;           /* floats per global load of A (1, 2, 4)                          */
    int vwn;           /* floats per global load of B and per store of C (1, 2, 4)       */
    int sa, sb;        /* how the A / B tile reaches the arithmetic: 0 = operands read straight
                          from global memory, 1 = staged in LDS through registers,
                          2 = staged in LDS by LDS-direct loads (vw 1 or 4 only; k-fastest
                          tiles are stored XOR-swizzled instead of padded)                 */
    int pad;           /* 1 = pad the LDS rows of register-staged tiles by 4 floats
                          (bank-conflict-free fragment reads)                              */
    int kwi;           /* the KWG loop advances kwi at a time, body unrolled (2 or 8)     */
    int mfma;          /* 0 = per-thread register tile on the vector ALU,
                          1 = v_mfma_f32_32x32x2_f32 wave tiles,
                          2 = v_mfma_f32_16x16x4_f32 wave tiles                           */
    int grp;           /* 1 = XCD-aware workgroup-to-tile order, 0 = row-major order      */
    int sk;            /* split K: sk workgroups per tile of C, each summing a contiguous
                          1/sk of the K slabs into its own M x N plane of a library-owned
                          device workspace; a second kernel adds the planes in fixed order
                          and applies alpha and beta.  0 or 1 = no split.                  */
    int ns;            /* LDS buffers per staged tile: 2 (also meant by 0), 3 or 4; more than 2
                          needs every staged operand to use LDS-direct loads, which then
                          run ns - 1 K slabs ahead of the arithmetic                       */
    int ksw;           /* matrix-core variants: the workgroup's waves form ksw groups (1, also
                          meant by 0; 2; 4); each group multiplies 1/ksw of every K slab into
                          accumulators of its own for the whole tile, and the groups' sums are
                          added through LDS in group order.  Threads = mdimc * ndimc * ksw.      */
} sgemm_config;

/* What the generator knows about one compiled variant. */
typedef struct sgemm_kernel_info {
    int vgprs;         /* architected VGPRs per lane                                      */
    int agprs;         /* accumulation VGPRs per lane                                     */
    int sgprs;
    int lds_bytes;     /* static LDS per workgroup                                        */
    int scratch_bytes; /* private segment per lane; > 0 means register spills             */
    int code_bytes;    /* size of the code object                                         */
    int from_cache;    /* 1 = read from the on-disk cache, 0 = compiled now               */
    float compile_ms;
} sgemm_kernel_info;

/* Options of tune_ex(); zero-initialise and set what you need (0 = default). */
typedef struct tune_opts {
    int space;          /* SGEMM_SPACE_*; 0 = SGEMM_SPACE_FULL                            */
    int warmup;         /* minimum untimed launches per configuration; default 2          */
    int reps;           /* timed samples per configuration (median is kept); default 7    */
    int verify_off;     /* 1 = skip the comparison against the reference kernel           */
    float cut_factor;   /* stop timing a configuration whose first sample is slower than
                           cut_factor x the best so far and keep that sample as its time;
                           default 3, negative = never cut                                 */
    float warmup_ms;    /* keep launching untimed until about this much GPU time has passed
                           (the clock needs ~20 ms of load to settle); default 25,
                           negative = none beyond `warmup`                                 */
    float sa_T;         /* annealing temperature (paper: 2, 4, 6); default 4              */
    int sa_raw_ms;      /* 1 = t, t' in raw milliseconds; 0 = percent of best-so-far      */
    int pso_S;          /* swarm size (paper: 3, 6); default 3                            */
    float pso_alpha;    /* probability of a random value per dimension; default 0.4       */
    float pso_beta;     /* probability of the particle's own best; default 0              */
    float pso_gamma;    /* probability of the swarm's best; default 0.4                   */
    float random_fraction; /* random search: fraction of the space if budget <= 0, rounded
                              down to whole configurations (at least 1)                       */
    const float *A;     /* optional caller-owned DEVICE operands in the call's layout;    */
    const float *B;     /*   when A is null the library allocates seeded synthetic ones   */
    float *C;           /*   (C is overwritten; C_in is restored from C0 before each run) */
    const float *C0;    /* optional DEVICE copy of the initial C (needed when beta != 0)  */
    int lda, ldb, ldc;
    const char *log_path; /* optional HOST path: one JSON line appended per evaluation    */
    int warm_start;     /* 1 = annealing (and particle 0 of the swarm) starts at the
                           configuration the per-shape cache would use for this shape, if it
                           lies in the searched space, instead of at a random one; -(i+1) =
                           start at configuration i of the space (tune_replay too)           */
    int reserved[7];
} tune_opts;

typedef struct tune_result {
    sgemm_config best;
    float best_ms;       /* median milliseconds of the best configuration                  */
    float best_gflops;   /* 2*M*N*K / best_ms                                              */
    int best_index;      /* its index in the enumerated space                              */
    int evaluations;     /* distinct configurations timed                                  */
    int failed;          /* of those: failed to compile, spilled or failed verification    */
    int space_size;      /* valid configurations in the space                              */
    int evals_to_best;   /* evaluations made when the best was first timed                 */
    float total_ms;      /* wall time of the whole search                                  */
    float compile_ms;    /* of which kernel generation                                      */
    int reserved[6];
} tune_result;

/* ---- the GEMM call ------------------------------------------------------------------
 * C = alpha * op(A) * op(B) + beta * C   (first equation of the matrix-multiplication case
 * study; `layout` says how A and B are stored, see above).
 * 0 <= M, N, K <= 2^31 - 1025 (a size rounded up to a tile edge stays an int), else
 * SGEMM_E_BADARG.  M == 0 or N == 0: no-op.  K == 0 or alpha == 0: C = beta * C and A, B are
 * not read.  beta == 0: C is written without being read, so NaN/Inf in it do not propagate.
 * The variant is the cached best configuration for (M,N,K,layout).  On a miss the nearest tuned
 * shape of the same layout (every size within about a factor of 1.5) lends its configuration if
 * the call has that shape's launch geometry (the same grid of tiles, the same split of K), or if
 * the library's cost model finds no built-in template that fits the sizes better; else the
 * built-in default runs: the tuned winners serve as templates, and a two-parameter cost model
 * per template (sustained fraction of a CU's peak, fixed cost per launch) picks the one whose
 * tile grid fills the 256 CUs in the fewest rounds, with split K where tiles are few and K long.
 * This call never tunes.  A variant not yet in the kernel cache is compiled on first use.
 * Large problems whose sizes are not multiples of the tile AND whose stored rows are not
 * multiples of the load vector go through zero-padded copies (sgemm_run_config_padded(); see
 * sgemm_config_prefers_padding()).
 * Device workspaces (split-K planes, padded copies) belong to the library, one set per stream,
 * allocated on first need and kept: calls on different streams never share one, calls on one
 * stream are ordered by the stream.  A call whose shape, leading dimensions, pointer alignment
 * and "beta is zero" have been seen before finds its loaded variant and launch plan by one hash
 * lookup; the first such call resolves, loads (compiles, if need be) and plans.
 * sgemm_tuned() launches on the stream given to sgemm_set_stream() (default: null stream). */
int sgemm_tuned(int M, int N, int K, float alpha, const float *A, int lda, const float *B,
                int ldb, float beta, float *C, int ldc, int layout);
int sgemm_tuned_on(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                   const float *B, int ldb, float beta, float *C, int ldc, int layout);
int sgemm_set_stream(void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same operation and the same variant as
 * sgemm_tuned_on(), with no hipMalloc, hipFree, module load or other allocating call inside.
 *   - The call must have been prepared: an earlier sgemm_tuned_on() call with the same M, N, K,
 *     layout, leading dimensions, pointer alignment (16 / 8 / 4 bytes, per operand) and the same
 *     "beta == 0" has loaded the variant.  Otherwise SGEMM_E_NOTREADY and nothing is launched.
 *   - Split-K planes lie in a statically allocated device array of SGEMM_NOALLOC_SCRATCH_BYTES
 *     (one per GPU, held until the process ends) instead of an allocated workspace.  A call whose
 *     planes (parts * M * N floats, see sgemm_config_workspace_bytes()) do not fit returns
 *     SGEMM_E_RESOURCE and launches nothing.  Every plane element that is read is written by the
 *     same call first, so nothing needs clearing between calls.
 *   - Zero-padded copies are never used: sizes that are not multiples of the tile run the
 *     guarded build (same result within rounding).
 *   - All calls on one GPU share that GPU's array: calls that split K and overlap in time (on
 *     different streams) race.  Order them, or use sgemm_tuned_on() for all but one stream.
 *   - The first call on a device looks up the array's device address (no allocation, but not
 *     capturable): make one call outside any graph capture first. */
#define SGEMM_NOALLOC_SCRATCH_BYTES (32u << 20)
int sgemm_tuned_noalloc(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                        const float *B, int ldb, float beta, float *C, int ldc, int layout);

/* The same call with on-line tuning (the paper's other mode of use: tuning "at run time, in the
 * first calls", section "CLTune: an auto-tuner for OpenCL kernels").  While (M,N,K,layout) has
 * no entry in the per-shape cache, every call computes its GEMM with the next configuration
 * that `strategy` proposes in `space` and times that one launch (the call then returns only when
 * the launch has finished); after `budget` distinct configurations the fastest one is put into
 * the cache and all later calls are ordinary asynchronous sgemm_tuned_on() calls.  Every call
 * returns a correct C.  A configuration that fails to compile, spills or fails to launch counts
 * as evaluated and the same call goes on to the next one.  Candidates are timed once, cold, and
 * are not re-verified against the reference kernel: a quick, noisy search compared with tune().
 * Host threads may make calls of one shape at the same time while it is being tuned: each
 * candidate is handed to exactly one call, the others wait for the next one (or for the end of
 * the search) and every call still computes its own GEMM; the times measured then include
 * whatever else the device was doing, as with any concurrent use. */
int sgemm_tuned_online(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                       const float *B, int ldb, float beta, float *C, int ldc, int layout,
                       int space, int strategy, int budget);

/* Same operation with an explicit configuration (what the tuner times and the parity tests
 * drive).  Returns SGEMM_E_INVALID if `cfg` breaks a constraint; picks the guarded-edge
 * build of the variant when M, N, K are not multiples of the tile, and narrows vwm/vwn to 1
 * when a pointer or leading dimension is not aligned for the vector width. */
int sgemm_run_config(void *hip_stream, const sgemm_config *cfg, int M, int N, int K,
                     float alpha, const float *A, int lda, const float *B, int ldb, float beta,
                     float *C, int ldc, int layout);

/* The same with the paper's pre-processing step instead of guarded builds (matrix-multiplication
 * case study: a "pre-processing kernel" makes the sizes multiples of the tile): A, B and, when
 * beta != 0, C are copied into zero-padded buffers of a library-owned device workspace whose
 * sizes are multiples of cfg's tile, the unguarded build runs on those, and the M x N result is
 * copied back into C.  Same result as sgemm_run_config() within rounding (the padding adds exact
 * zeros); four extra kernels and (|A| + |B| + 2|C|) of extra traffic.  Sizes that already are
 * multiples take the ordinary path.  The workspace belongs to the stream of the call. */
int sgemm_run_config_padded(void *hip_stream, const sgemm_config *cfg, int M, int N, int K,
                            float alpha, const float *A, int lda, const float *B, int ldb, float beta,
                            float *C, int ldc, int layout);

/* [host] Whether sgemm_tuned() / sgemm_tuned_on() would take the padded path for this call with
 * cfg (pointers assumed 16-byte aligned): 1 when the sizes are not multiples of cfg's tile, a
 * stored row is not a multiple of the load vector (so the guarded build would load pairs or
 * single floats) and the problem is large enough for the copies to pay, by a model fitted to
 * measurements (odd row lengths: cubes from about 3800 for beta = 0, 4900 for beta != 0; even
 * row lengths keep 2-float loads and are not padded at any measured size); else 0.  The tuner and sgemm_run_config() never pad
 * on their own. */
int sgemm_config_prefers_padding(const sgemm_config *cfg, int M, int N, int K, int lda, int ldb, int ldc,
                                 int layout, float beta);

/* The reference kernel every tested configuration is compared with inside tune*() (the
 * paper's result verification, section "Advanced usage"): one thread per element of C,
 * products and sums in double, result rounded to float.  Exported so that tests can check it. */
int sgemm_reference(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                    const float *B, int ldb, float beta, float *C, int ldc, int layout);

/* ---- tuning -------------------------------------------------------------------------
 * tune(): search the full space for (M,N,K), row-major A and B, alpha = 1, beta = 0, on
 * library-owned synthetic operands; store the winner in the per-shape cache.  `strategy` is
 * SGEMM_STRATEGY_*; `budget` = maximum number of distinct configurations timed (ignored by
 * the full search).  Returns the number of configurations evaluated (>= 0) or an error.
 * tune_ex(): the same with everything explicit; fills *out (may be null). */
int tune(int M, int N, int K, int strategy, int budget);
int tune_ex(int M, int N, int K, int layout, float alpha, float beta, int strategy, int budget,
            unsigned long long seed, const tune_opts *opts, tune_result *out);

/* [host] Run a strategy against a table of known costs instead of the GPU: ms_table[i] is
 * the time of configuration i of `space` (a non-finite or non-positive entry marks a failed
 * configuration).  visited (may be null) receives up to visited_cap configuration indices in
 * evaluation order.  This is how recorded full searches are replayed for strategy studies
 * (the paper repeats every search 128 times).  Returns evaluations made or an error. */
int tune_replay(int space, const float *ms_table, int table_len, int strategy, int budget,
                unsigned long long seed, const tune_opts *opts, int *visited, int visited_cap,
                tune_result *out);

/* ---- search space [host] ------------------------------------------------------------- */
/* Define SGEMM_SPACE_CUSTOM, the counterpart of the paper's AddParameter(name, {values}) for this
 * kernel family ("CLTune: an auto-tuner for OpenCL kernels"): `spec` is HOST text of the form
 * "MWG=64,128 NWG=128 KWG=32,64 SK=4,8" - parameter names as in sgemm_config (upper case),
 * separated by blanks or ';'.  A parameter that is not named keeps one value (MWG=NWG=128 KWG=32
 * MDIMC=NDIMC=16 VWM=VWN=4 SA=SB=1 PAD=1 KWI=8 MFMA=1 GRP=0 SK=1 NS=2 KSW=1).  The product is pruned by
 * the kernel family's constraints like every preset.  Returns the number of valid
 * configurations (>= 0) or SGEMM_E_BADARG.  A process that never calls this reads the
 * definition from $SGEMM_TUNED_CUSTOM_SPACE on first use.  Redefining the space while a search
 * over it runs is safe; that search finishes on the old definition. */
int sgemm_space_define_custom(const char *spec);
int sgemm_space_size(int space);      /* valid configurations after constraint pruning     */
long long sgemm_space_raw_size(int space); /* plain product of the value-list lengths      */
int sgemm_space_get(int space, int index, sgemm_config *out);
int sgemm_space_find(int space, const sgemm_config *cfg); /* index, or SGEMM_E_INVALID     */
int sgemm_space_dims(int space);      /* number of tuned parameters                        */
/* values of parameter `dim` (0-based, in sgemm_config field order); returns the count */
int sgemm_space_values(int space, int dim, int *values, int cap);
/* SGEMM_OK if cfg satisfies every constraint of the kernel family (divisibility, thread
 * count, register budget, LDS capacity), else SGEMM_E_INVALID. */
int sgemm_config_check(const sgemm_config *cfg);
int sgemm_config_lds_bytes(const sgemm_config *cfg); /* LDS the variant will declare       */
int sgemm_config_default(int M, int N, int K, int layout, sgemm_config *out);
/* How cfg's split K applies to a problem with this K: *parts (may be null) receives the number
 * of workgroups per tile that will really be launched (sk limited to the number of K slabs,
 * no empty parts), *k_chunk (may be null) the k range of each part, a multiple of kwg (K itself
 * when there is one part).  Returns the bytes of device workspace a call with this
 * configuration uses for an M x N result: parts * M * N * 4, or 0 when parts == 1. */
long long sgemm_config_workspace_bytes(const sgemm_config *cfg, int M, int N, int K, int *parts,
                                       int *k_chunk);

/* ---- kernel generator --------------------------------------------------------------- */
/* [host] Directory of the on-disk code-object cache (default: "kcache" beside the library,
 * or $SGEMM_TUNED_CACHE_DIR). */
int sgemm_kernel_cache_dir(const char *path);
/* Builds of one configuration (the `build` argument below is a sum of these flags):
 * guarded against sizes that are not multiples of the tile, and - for calls with beta != 0 on
 * the matrix-core schedule, where a lane has the registers for it - requesting the old values
 * of C before the main loop instead of in the epilogue. */
#define SGEMM_BUILD_GUARDED 1
#define SGEMM_BUILD_READS_C_AHEAD 2
/* [host] Compile (or fetch from the cache) the variant for cfg/layout in the given build
 * (0 = plain, 1 = SGEMM_BUILD_GUARDED as before).  cfg must satisfy every constraint but the register estimate (the build
 * that sgemm_kernel_resolve() names may have narrower load vectors than the configuration it
 * came from and then exceeds the estimate; it still has to be built).  cfg->sk > 1 selects the build that split-K launches use (one build
 * for every sk > 1: the split itself is a launch parameter).  Needs no GPU.  info may be null. */
int sgemm_kernel_compile(const sgemm_config *cfg, int layout, int build, sgemm_kernel_info *info);
/* [host] Which build a call with cfg launches for these sizes, leading dimensions and beta
 * (only beta == 0 or not matters) when the operands' pointers are 16-byte aligned: *variant
 * receives the configuration as it is built (vector widths narrowed where a stored row is not
 * a multiple of them, fewer LDS buffers or register staging where narrowed LDS-direct loads no
 * longer fit, sk = 1 when K is not split) and *build the SGEMM_BUILD_* flags, so that
 * sgemm_kernel_compile(variant, layout, *build) prepares exactly what the call will load. */
int sgemm_kernel_resolve(const sgemm_config *cfg, int M, int N, int K, int lda, int ldb, int ldc,
                         int layout, float beta, sgemm_config *variant, int *build);
/* [host] Path of the variant's code object in the cache directory (whether or not it exists
 * yet), NUL-terminated into buf: lets a deployment ship exactly the variants it uses. */
int sgemm_kernel_cache_path(const sgemm_config *cfg, int layout, int build, char *buf, int cap);
/* [host] The -D macro string the variant is compiled with, NUL-terminated into buf. */
int sgemm_kernel_macros(const sgemm_config *cfg, int layout, int build, char *buf, int cap);

/* ---- per-shape best-configuration cache --------------------------------------------- */
int sgemm_config_get(int M, int N, int K, int layout, sgemm_config *out); /* exact shape only;
                                         SGEMM_E_NOCONFIG on a miss */
int sgemm_config_set(int M, int N, int K, int layout, const sgemm_config *cfg, float ms);
int sgemm_config_select(int M, int N, int K, int layout, sgemm_config *out); /* what
                                         sgemm_tuned() would use: exact, nearest, default */
int sgemm_cache_load(const char *path); /* merge a text file into the cache               */
int sgemm_cache_save(const char *path);
int sgemm_cache_clear(void);
int sgemm_cache_count(void);

/* ---- device facts ------------------------------------------------------------------- */
/* FP32 peak in GFLOP/s = compute units x 256 FLOP/clk x clock, from the device's own
 * properties; also returns CU count and clock (MHz) if the pointers are non-null. */
int sgemm_device_peak(float *gflops, int *compute_units, int *clock_mhz);

const char *sgemm_status_string(int status);
/* Detail of the calling thread's most recent failure (compiler log, HIP error string); the
 * pointer stays valid until that thread's next failing call.  Never null. */
const char *sgemm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SGEMM_TUNED_H */
