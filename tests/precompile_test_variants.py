"""Put every kernel variant that tests/test_gpu_parity.py launches into the on-disk kernel
cache, in parallel and without a GPU, so that the GPU run spends no time compiling:

    python tests/precompile_test_variants.py

(The tests pass without this step; they then compile each variant on first use.)"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from paper_1703_06503_amd import binding as b            # noqa: E402
from tests import test_gpu_parity as t                   # noqa: E402


def tuned_table_variants():
    """The variants that sgemm_tuned() launches for the shapes of the committed table of tuned
    configurations (what bench.py, smoke() and the full-size tests run)."""
    from paper_1703_06503_amd import report
    table = os.path.join(os.path.dirname(b.LIB_PATH), "..", "tuned_configs.txt")
    for M, N, K, layout, _ms, cfg in report.read_table(table):
        c = b.make_config(*cfg)
        edge = 1 if (M % c.mwg or N % c.nwg or K % c.kwg) else 0
        b.sgemm_kernel_compile(c, layout, edge)


def fixed_config_variants():
    """The hand-picked configurations of the parity tests, in every layout, guarded and not."""
    for cfg in t._some_configs():
        for layout in (0, 1, 2, 3):
            for edge in (0, 1):
                b.sgemm_kernel_compile(cfg, layout, edge)
        M, N, K = t.NARROW_SHAPE
        for layout in (0, 3):
            variant, edge = b.sgemm_kernel_resolve(cfg, M, N, K, M if layout & 1 else K, K if layout & 2 else N, N, layout)
            b.sgemm_kernel_compile(variant, layout, edge)


def conv_variants():
    """The convolution variants of tests/test_gpu_conv.py: guarded and unguarded, with and
    without vector accesses (which of the four a call uses depends on sizes and alignment)."""
    from tests import test_gpu_conv as tc
    todo = []
    for (Xf, Yf) in tc.SAMPLES:
        todo += [(b.conv2d_space_get(Xf, Yf, i), Xf, Yf) for i in tc.sample(Xf, Yf)]
    for c in tc.CONFIGS:
        todo += [(b.make_conv_config(*c), f[0], f[1]) for f in ((7, 5), (3, 3))]
    b.conv2d_cache_clear()
    for fx, fy in [(3, 3), (5, 5), (7, 7), (11, 11), (1, 1), (2, 5), (9, 9), (11, 3), (13, 13), (31, 5), (17, 17)]:
        todo.append((b.conv2d_config_select(1, 1, fx, fy)[1], fx, fy))
    for cfg, Xf, Yf in todo:
        for edge in (0, 1):
            for vector in (0, 1):
                b.conv2d_kernel_compile(cfg, Xf, Yf, edge, vector)


def _resolve_and_compile(task):
    space, index, (M, N, K), layout = task
    cfg = b.sgemm_space_get(space, index)
    lda = M if layout & 1 else K
    ldb = K if layout & 2 else N
    variant, edge = b.sgemm_kernel_resolve(cfg, M, N, K, lda, ldb, N, layout)
    return 0 if b.sgemm_kernel_compile(variant, layout, edge).from_cache else 1


def sweep_variants(jobs):
    """Exactly the build each case of the parity sweeps loads: which one that is depends on the
    sizes too (vector widths are narrowed where a stored row is not a multiple of them)."""
    import multiprocessing as mp
    tasks = [(space, i, shape, layout) for space, idx, shape, layout in t.all_sweeps() for i in idx]
    with mp.get_context("spawn").Pool(jobs) as pool:
        new = sum(pool.map(_resolve_and_compile, tasks, chunksize=8))
    print(f"parity sweeps: {len(tasks)} cases, {new} variants compiled now", flush=True)


def main():
    jobs = min(8, os.cpu_count() or 1)
    tuned_table_variants()
    fixed_config_variants()
    conv_variants()
    sweep_variants(jobs)
if __name__ == "__main__":
    main()
