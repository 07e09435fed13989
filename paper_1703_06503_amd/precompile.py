"""Fill the on-disk code-object cache ahead of time, in parallel, without a GPU:

    python -m paper_1703_06503_amd.precompile --space 0 --layouts 0 --edge 0 --jobs 8

Recompilation can dominate tuning time (paper, section "Search strategies and search-space
properties"); compiling every variant of a space once, off-line, takes it out of the search."""
import argparse
import multiprocessing as mp
import sys
import time


def _work(args):
    space, layout, edge, lo, hi, step, beta = args
    from . import binding as b
    n_new = n_fail = 0
    for i in range(lo, hi, step):
        cfg = b.sgemm_space_get(space, i)
        try:
            if isinstance(edge, tuple):     # a problem shape: the build a call of that shape loads
                M, N, K = edge
                cfg, e = b.sgemm_kernel_resolve(cfg, M, N, K, M if layout & 1 else K, K if layout & 2 else N,
                                                N, layout, beta)
            else:
                e = edge
            info = b.sgemm_kernel_compile(cfg, layout, e)
            n_new += 0 if info.from_cache else 1
        except b.SgemmError:
            n_fail += 1
    return n_new, n_fail


def precompile(space=0, layouts=(0,), edges=(0,), jobs=8, indices=None, verbose=True, beta=0.0):
    from . import binding as b
    n = b.sgemm_space_size(space)
    t0 = time.time()
    total_new = total_fail = 0
    ctx = mp.get_context("spawn")
    with ctx.Pool(jobs) as pool:
        for layout in layouts:
            for edge in edges:
                if indices is None:
                    indices_now = range(n)
                else:
                    indices_now = indices
                # small strided chunks, so that progress can be reported while the pool works
                chunks = max(jobs * 8, len(indices_now) // 16)
                tasks = [(space, layout, edge, j, len(indices_now), chunks, beta) for j in range(chunks)]
                if indices is not None:
                    tasks = [(space, layout, edge, i, i + 1, 1, beta) for i in indices]
                last = time.time()
                for done, r in enumerate(pool.imap_unordered(_work, tasks), 1):
                    total_new += r[0]
                    total_fail += r[1]
                    if verbose and time.time() - last > 20:
                        last = time.time()
                        print(f"  {done}/{len(tasks)} chunks, compiled {total_new}, {time.time() - t0:.0f} s", flush=True)
                if verbose:
                    print(f"space {space} layout {layout} edge {edge}: compiled so far "
                          f"{total_new}, failed {total_fail}, {time.time() - t0:.0f} s", flush=True)
    return total_new, total_fail


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--space", type=int, default=0)
    ap.add_argument("--layouts", default="0")
    ap.add_argument("--edge", default="0")
    ap.add_argument("--jobs", type=int, default=8)
    ap.add_argument("--shape", default=None,
                    help="M,N,K: compile for each configuration the build that a call of this shape "
                         "loads (guarded or not, load vectors narrowed where rows demand it, the "
                         "split-K build where K is split) instead of --edge")
    ap.add_argument("--beta", type=float, default=0.0,
                    help="with --shape: the calls' beta (builds for beta != 0 may differ)")
    ap.add_argument("--values", default=None,
                    help='value lists of the caller-defined space (--space 5), e.g. "MWG=64,128 SK=4,8"')
    a = ap.parse_args(argv)
    if a.values:
        import os
        os.environ["SGEMM_TUNED_CUSTOM_SPACE"] = a.values      # the worker processes read it
    edges = [tuple(int(x) for x in a.shape.split(","))] if a.shape else [int(x) for x in a.edge.split(",")]
    new, fail = precompile(a.space, [int(x) for x in a.layouts.split(",")], edges, a.jobs, beta=a.beta)
    print(f"compiled {new} variants, {fail} failed")
    return 1 if fail else 0


if __name__ == "__main__":
    sys.exit(main())
