"""Command-line front end for the second kernel family, the tunable 2D convolution
(paper: "Case-study: 2D convolution").

    python -m paper_1703_06503_amd.conv_cli precompile --filter 7 --jobs 8     # no GPU needed
    python -m paper_1703_06503_amd.conv_cli tune --workload conv_7x7 --strategy full --log conv7.jsonl
    python -m paper_1703_06503_amd.conv_cli run --workload conv_7x7 --config 32,8,2,4,1,2,0,1
    python -m paper_1703_06503_amd.conv_cli cross conv_3x3 conv_7x7 conv_11x11 --configs ...

`tune` searches the space of the workload's filter with the library's tuner and appends one JSON
line per evaluated configuration to --log (the record `strategy_study --space conv7x7` replays).
`run` times one configuration, or with no --config the library's choice, on the workload's seeded
image and reports the paper's two figures: GFLOP/s = (1 + 2 Xf Yf) X Y / t and GB/s = 2 X Y floats
/ t.  `cross` is the paper's table "Merits of filter size tuning": every workload run with the
configuration given for each of them."""
import argparse
import multiprocessing as mp
import statistics
import sys
import time

STRATEGIES = {"full": 0, "random": 1, "annealing": 2, "pso": 3}


def _compile_range(args):
    Xf, Yf, lo, hi, step, edge = args
    from . import binding as b
    fail = 0
    for i in range(lo, hi, step):
        try:
            b.conv2d_kernel_compile(b.conv2d_space_get(Xf, Yf, i), Xf, Yf, edge, 1)
        except b.SgemmError:
            fail += 1
    return fail


def precompile(Xf, Yf, jobs, edge=0):
    from . import binding as b
    n = b.conv2d_space_size(Xf, Yf)
    t0 = time.time()
    with mp.get_context("spawn").Pool(jobs) as pool:
        fail = sum(pool.map(_compile_range, [(Xf, Yf, j, n, jobs * 4, edge) for j in range(jobs * 4)]))
    print(f"{Xf}x{Yf}: {n} variants in the cache, {fail} failed, {time.time() - t0:.0f} s")
    return fail


def _device_inputs(w):
    import torch
    from . import synth
    A, F = synth.make_conv_workload(w)
    dA, dF = torch.from_numpy(A).cuda(), torch.from_numpy(F).cuda()
    dB = torch.empty((w.Y, w.X), dtype=torch.float32, device="cuda")
    return dA, dF, dB, A.shape[1]


def time_config(b, torch, cfg, w, dA, dF, dB, lda, reps=11, warm_ms=25.0):
    """Median milliseconds per call on resident operands (cfg None: the library's choice)."""
    def call():
        if cfg is None:
            b.conv2d_tuned(w.X, w.Y, w.Xf, w.Yf, w.w, dF, dA, lda, dB, w.X)
        else:
            b.conv2d_run_config(None, cfg, w.X, w.Y, w.Xf, w.Yf, w.w, dF, dA, lda, dB, w.X)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); call(); e1.record()
    torch.cuda.synchronize()
    first = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(min(4096, int(warm_ms / first) + 1)):
        call()
    batch = max(1, min(64, int(0.2 / first) + 1))
    samples = []
    for _ in range(reps):
        e0.record()
        for _ in range(batch):
            call()
        e1.record()
        torch.cuda.synchronize()
        samples.append(e0.elapsed_time(e1) / batch)
    return statistics.median(samples)


def figures(w, ms):
    """The paper's two figures of merit for a time in milliseconds."""
    return ((1 + 2 * w.Xf * w.Yf) * w.X * w.Y / ms * 1e-6, 2 * w.X * w.Y * 4 / ms * 1e-6)


def verified(b, torch, cfg, w, dA, dF, dB, lda):
    ref = torch.empty_like(dB)
    b.conv2d_reference(None, w.X, w.Y, w.Xf, w.Yf, w.w, dF, dA, lda, ref, w.X)
    dB.fill_(-1.0)
    if cfg is None:
        b.conv2d_tuned(w.X, w.Y, w.Xf, w.Yf, w.w, dF, dA, lda, dB, w.X)
    else:
        b.conv2d_run_config(None, cfg, w.X, w.Y, w.Xf, w.Yf, w.w, dF, dA, lda, dB, w.X)
    torch.cuda.synchronize()
    return bool((dB == ref).all())      # all variants add their taps in the reference's order


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("precompile")
    p.add_argument("--filter", type=int, nargs="+", default=[3, 7, 11])
    p.add_argument("--jobs", type=int, default=8)
    p.add_argument("--edge", type=int, default=0)
    p = sub.add_parser("tune")
    p.add_argument("--workload", required=True)
    p.add_argument("--strategy", choices=sorted(STRATEGIES), default="annealing")
    p.add_argument("--budget", type=int, default=0)
    p.add_argument("--fraction", type=float, default=0.0)
    p.add_argument("--seed", type=int, default=0)
    p.add_argument("--reps", type=int, default=0)
    p.add_argument("--warmup-ms", type=float, default=0.0)
    p.add_argument("--sa-T", type=float, default=0.0)
    p.add_argument("--pso-S", type=int, default=0)
    p.add_argument("--log", default=None)
    p.add_argument("--save", default=None, help="merge the winner into this table of best configurations")
    p = sub.add_parser("run")
    p.add_argument("--workload", required=True)
    p.add_argument("--config", default=None)
    p = sub.add_parser("cross")
    p.add_argument("workloads", nargs="+")
    p.add_argument("--configs", nargs="+", required=True,
                   help="one comma-separated configuration per workload, in the same order")
    a = ap.parse_args(argv)

    from . import binding as b
    from . import synth
    if a.cmd == "precompile":
        return 1 if sum(precompile(f, f, a.jobs, a.edge) for f in a.filter) else 0

    import torch
    if a.cmd == "tune":
        w = synth.CONV_WORKLOADS[a.workload]
        o = b.tune_opts()
        o.reps, o.warmup_ms, o.sa_T, o.pso_S, o.random_fraction = a.reps, a.warmup_ms, a.sa_T, a.pso_S, a.fraction
        if a.log:
            o.log_path = a.log.encode()
        if a.save:
            import os
            if os.path.exists(a.save):
                b.conv2d_cache_load(a.save)
        n, res = b.conv2d_tune(w.X, w.Y, w.Xf, w.Yf, w.w, STRATEGIES[a.strategy], a.budget, a.seed, o)
        if a.save:
            b.conv2d_cache_save(a.save)
        print(f"{a.workload}: {n} of {res.space_size} configurations evaluated ({res.failed} failed) in "
              f"{res.total_ms / 1e3:.1f} s (compiling {res.compile_ms / 1e3:.1f} s); best "
              f"{','.join(map(str, res.best.as_tuple()))}: {res.best_ms:.4f} ms = {res.best_gflops:.0f} GFLOP/s, "
              f"{res.best_gbs:.0f} GB/s; found after {res.evals_to_best} evaluations")
        return 0
    if a.cmd == "run":
        w = synth.CONV_WORKLOADS[a.workload]
        cfg = b.make_conv_config(*[int(x) for x in a.config.split(",")]) if a.config else None
        dA, dF, dB, lda = _device_inputs(w)
        if not verified(b, torch, cfg, w, dA, dF, dB, lda):
            print("result differs from the reference kernel", file=sys.stderr)
            return 1
        ms = time_config(b, torch, cfg, w, dA, dF, dB, lda)
        gf, gb = figures(w, ms)
        used = cfg or b.conv2d_config_select(w.X, w.Y, w.Xf, w.Yf)[1]
        print(f"{a.workload} {','.join(map(str, used.as_tuple()))}: {ms:.4f} ms, {gf:.0f} GFLOP/s, {gb:.0f} GB/s")
        return 0
    # cross
    ws = [synth.CONV_WORKLOADS[n] for n in a.workloads]
    cfgs = [b.make_conv_config(*[int(x) for x in c.split(",")]) for c in a.configs]
    if len(cfgs) != len(ws):
        ap.error("one configuration per workload")
    ms = {}
    for w in ws:
        dA, dF, dB, lda = _device_inputs(w)
        for src, cfg in zip(ws, cfgs):
            if b.conv2d_config_check(cfg, w.Xf, w.Yf) != b.OK:
                ms[w.name, src.name] = None
                continue
            if not verified(b, torch, cfg, w, dA, dF, dB, lda):
                print(f"{src.name}'s configuration fails on {w.name}", file=sys.stderr)
                return 1
            ms[w.name, src.name] = time_config(b, torch, cfg, w, dA, dF, dB, lda)
    print("| applied to \\ best parameters for | " + " | ".join(w.name for w in ws) + " |")
    print("|---|" + "---|" * len(ws))
    for w in ws:
        own = min(t for (r, _), t in ms.items() if r == w.name and t)
        cells = []
        for s in ws:
            t = ms[w.name, s.name]
            cells.append("invalid" if t is None else f"{t:.4f} ms ({100 * own / t:.0f} %)")
        print(f"| {w.name} | " + " | ".join(cells) + " |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
