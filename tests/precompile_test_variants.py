"""Put every kernel variant that the GPU tests, smoke() and bench.py launch into the on-disk
kernel cache, in parallel worker processes and without a GPU (the kernel generator needs none),
so that a GPU run compiles nothing:

    python tests/precompile_test_variants.py [jobs]

Variants already in the cache are skipped, so a second run costs seconds.  (The tests also pass
without this step; they then compile each variant on first use.)"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from paper_1703_06503_amd import binding as b            # noqa: E402
from tests import variants as v                          # noqa: E402

PLANTED_BUG = "-DPLANT_SKIP_TILE=1"   # tests/test_gpu_parity.py: verification must notice it


def _gemm(cfg, layout, edge, extra=""):
    return ("gemm", cfg.as_tuple(), layout, edge, extra)


def _resolved(cfg, M, N, K, layout, pad=0):
    """The builds a call with cfg launches for these sizes (aligned pointers, stored rows `pad`
    floats longer than the matrices' rows): the one for beta == 0 and the one for beta != 0,
    which differ for some configurations."""
    lda, ldb = (M if layout & 1 else K) + pad, (K if layout & 2 else N) + pad
    out = []
    for beta in (0.0, 1.0):
        variant, build = b.sgemm_kernel_resolve(cfg, M, N, K, lda, ldb, N, layout, beta)
        out.append(_gemm(variant, layout, build))
    return out


def gemm_tasks():
    from paper_1703_06503_amd import report, synth
    tasks = []
    # the committed table of tuned configurations: what sgemm_tuned() launches for its shapes
    table = os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt")
    b.sgemm_cache_clear()
    b.sgemm_cache_load(table)
    for M, N, K, layout, _ms, cfg in report.read_table(table):
        tasks += _resolved(b.make_config(*cfg), M, N, K, layout)
    # configurations run at the benchmark sizes beside the winners
    for name in ("cfg4_4096", "cfg2_2048", "cfg3_1000", "cfg3_1536"):
        w = synth.WORKLOADS[name]
        tasks += [t for cfg in v.BENCH_CONFIGS for t in _resolved(cfg, w.M, w.N, w.K, w.layout)]
    for name in ("cfg5_128x4096x4096", "cfg5_4096x64x9216"):
        w = synth.WORKLOADS[name]
        tasks += [t for cfg in v.SKINNY_CONFIGS for t in _resolved(cfg, w.M, w.N, w.K, w.layout)]
    # dispatch without an exactly tuned shape; the pad-and-run path loads the unguarded build
    for M, N, K, layout in v.DISPATCHED_CALLS + [c[:4] for c in v.NOALLOC_CALLS]:
        cfg = b.sgemm_config_select(M, N, K, layout)
        tasks += _resolved(cfg, M, N, K, layout) + [_gemm(cfg, layout, 0), _gemm(cfg, layout, b.BUILD_READS_C_AHEAD)]
    (M, N, K, layout), cfg = v.NOALLOC_TOO_BIG
    tasks += _resolved(cfg, M, N, K, layout)
    # the hand-picked configurations, in every layout, guarded and not, and narrowed
    for cfg in v.some_configs():
        tasks += [_gemm(cfg, layout, build) for layout in (0, 1, 2, 3) for build in (0, 1, 2, 3)]
        tasks += [t for layout in (0, 3) for t in _resolved(cfg, *v.NARROW_SHAPE, layout)]
        for shape in [(97, 83, 45), (130, 70, 33), (1, 1, 1), (5, 300, 2), (200, 100, 300), (150, 140, 60),
                      (192, 160, 192), (384, 256, 512), (300, 200, 150)]:
            tasks += _resolved(cfg, *shape, 0)
    # tests/test_gpu_parity.py: NaN frames around the operands, rows 4 MiB apart
    for which in (0, 1, 3, 4, 6, 10):
        for layout in (0, 1, 2, 3):
            for shape, pad in [((97, 83, 45), 3), ((150, 140, 60), 4), ((64, 64, 64), 8)]:
                tasks += _resolved(v.some_configs()[which], *shape, layout, pad)
    for cfg in (v.some_configs()[1], v.some_configs()[4], b.make_config(256, 256, 32, 32, 8, 4, 4, 1, 1, 0, 8, 1, 0, 1, 2)):
        tasks += _resolved(cfg, 200, 72, 40, 0, (1 << 20) - 72)     # ldb = 2^20; lda is as aligned as 2^20 is
    for cfg in v.ODD_EDGE_CONFIGS:
        tasks += [t for shape in v.ODD_EDGE_SHAPES for layout in (0, 1, 2, 3) for t in _resolved(cfg, *shape, layout)]
    # the sweeps: which build a case loads depends on the sizes too
    for space, idx, shape, layout in v.all_sweeps():
        tasks += [t for i in idx for t in _resolved(b.sgemm_space_get(space, i), *shape, layout)]
    # the small space: the tuner tests search it on several shapes, once with the planted bug
    for i in range(b.sgemm_space_size(b.SPACE_SMALL)):
        cfg = b.sgemm_space_get(b.SPACE_SMALL, i)
        tasks.append(_gemm(cfg, 0, 0, PLANTED_BUG))
        tasks += [t for shape in [(192, 160, 96), (256, 256, 128), (320, 256, 192)] for t in _resolved(cfg, *shape, 0)]
    return tasks


def conv_tasks():
    """The convolution variants of tests/test_gpu_conv.py: guarded and unguarded, with and
    without vector accesses (which of the four a call uses depends on sizes and alignment)."""
    todo = []
    for (Xf, Yf) in v.CONV_SAMPLES:
        todo += [(b.conv2d_space_get(Xf, Yf, i), Xf, Yf) for i in v.conv_sample(Xf, Yf)]
    for c in v.CONV_CONFIGS:
        todo += [(b.make_conv_config(*c), f[0], f[1]) for f in ((7, 5), (3, 3))]
    b.conv2d_cache_clear()
    for fx, fy in v.CONV_DEFAULT_FILTERS:
        todo.append((b.conv2d_config_select(1, 1, fx, fy)[1], fx, fy))
    return [("conv", cfg.as_tuple(), Xf, Yf, edge, vector)
            for cfg, Xf, Yf in todo for edge in (0, 1) for vector in (0, 1)]


def _compile(task):
    """1 if the variant was compiled now, 0 if it was in the cache already; a failure comes back
    as text (an exception raised in a pool worker must not be left to the pool to carry)."""
    try:
        return _compile_task(task)
    except Exception as e:      # noqa: BLE001
        return f"{task}: {e}"


def _compile_task(task):
    if task[0] == "gemm":
        _, cfg, layout, edge, extra = task
        if extra:
            os.environ["SGEMM_TUNED_EXTRA_DEFINES"] = extra
        else:
            os.environ.pop("SGEMM_TUNED_EXTRA_DEFINES", None)
        info = b.sgemm_kernel_compile(b.make_config(*cfg), layout, edge)
    else:
        _, cfg, Xf, Yf, edge, vector = task
        info = b.conv2d_kernel_compile(b.make_conv_config(*cfg), Xf, Yf, edge, vector)
    return 0 if info.from_cache else 1


def main(jobs=None, verbose=True):
    import multiprocessing as mp
    jobs = jobs or min(8, os.cpu_count() or 1)
    tasks = sorted(set(gemm_tasks() + conv_tasks()))
    with mp.get_context("spawn").Pool(jobs) as pool:
        results = pool.map(_compile, tasks, chunksize=4)
    failures = [r for r in results if isinstance(r, str)]
    if failures:
        raise RuntimeError(f"{len(failures)} variants failed to compile, the first: {failures[0]}")
    new = sum(results)
    if verbose:
        print(f"kernel cache: {len(tasks)} variants wanted, {new} compiled now", flush=True)
    return len(tasks), new


if __name__ == "__main__":
    main(int(sys.argv[1]) if len(sys.argv) > 1 else None)
