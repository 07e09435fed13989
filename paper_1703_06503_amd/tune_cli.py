"""Command-line front end of the tuner: tune one benchmark workload on its seeded operands.

    python -m paper_1703_06503_amd.tune_cli --workload cfg2_2048 --strategy full \\
        --space full --log results/cfg2_full.jsonl --save results/tuned_configs.txt

Every evaluated configuration is appended to --log as one JSON line (configuration, status,
median ms, GFLOP/s, registers, LDS), which is also the record that strategy studies replay
(`tune_replay`).  --save writes the per-shape best-configuration table."""
import argparse
import json
import sys
import time

STRATEGIES = {"full": 0, "random": 1, "annealing": 2, "pso": 3}
SPACES = {"full": 0, "small": 1, "mfma": 2, "ext": 3, "direct": 4, "custom": 5, "ksplit": 6}


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--strategy", choices=sorted(STRATEGIES), default="pso")
    ap.add_argument("--space", choices=sorted(SPACES), default="full")
    ap.add_argument("--values", default=None,
                    help='value lists of --space custom, e.g. "MWG=64,128 NWG=128 SK=4,8"')
    ap.add_argument("--budget", type=int, default=0)
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--reps", type=int, default=0)
    ap.add_argument("--warmup-ms", type=float, default=0.0)
    ap.add_argument("--cut-factor", type=float, default=0.0)
    ap.add_argument("--sa-T", type=float, default=0.0)
    ap.add_argument("--pso-S", type=int, default=0)
    ap.add_argument("--fraction", type=float, default=0.0)
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--warm-start", action="store_true",
                    help="start annealing / particle 0 at the configuration cached for the shape")
    ap.add_argument("--log", default=None)
    ap.add_argument("--save", default=None)
    ap.add_argument("--load", default=None, help="best-configuration table to merge first")
    ap.add_argument("--start-config", default=None,
                    help="comma-separated configuration (field order of sgemm_config) to put into "
                         "the per-shape cache for this workload before the search; with "
                         "--warm-start the search begins there")
    a = ap.parse_args(argv)

    import torch
    from . import binding as b
    from . import synth

    w = synth.WORKLOADS[a.workload]
    A, B, C = synth.make_workload(w)
    dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
    dC = dC0.clone()
    if a.load:
        b.sgemm_cache_load(a.load)
    if a.start_config:
        start = b.make_config(*[int(x) for x in a.start_config.split(",")])
        b.sgemm_config_set(w.M, w.N, w.K, w.layout, start, 0.0)   # time unknown: any result replaces it
    if a.space == "custom":
        if not a.values:
            ap.error("--space custom needs --values")
        print(f"custom space: {b.sgemm_space_define_custom(a.values)} valid configurations", file=sys.stderr)
    opts = b.tune_opts()
    opts.space = SPACES[a.space]
    opts.reps = a.reps
    opts.warmup_ms = a.warmup_ms
    opts.cut_factor = a.cut_factor
    opts.sa_T = a.sa_T
    opts.pso_S = a.pso_S
    opts.random_fraction = a.fraction
    opts.verify_off = 1 if a.no_verify else 0
    opts.warm_start = 1 if a.warm_start else 0
    opts.A, opts.B, opts.C, opts.C0 = dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), dC0.data_ptr()
    opts.lda, opts.ldb, opts.ldc = A.shape[1], B.shape[1], w.N
    if a.log:
        opts.log_path = a.log.encode()
    seed = w.seed if a.seed is None else a.seed
    t0 = time.time()
    evals, res = b.tune_ex(w.M, w.N, w.K, w.layout, w.alpha, w.beta, STRATEGIES[a.strategy],
                           a.budget, seed, opts)
    peak, _, _ = b.sgemm_device_peak()
    summary = {
        "workload": a.workload, "strategy": a.strategy, "space": a.space, "budget": a.budget,
        "seed": seed, "evaluations": evals, "failed": res.failed, "space_size": res.space_size,
        "best_index": res.best_index, "best": res.best.as_dict(), "best_ms": res.best_ms,
        "best_gflops": res.best_gflops, "pct_peak": 100.0 * res.best_gflops / peak,
        "evals_to_best": res.evals_to_best, "seconds": time.time() - t0,
        "compile_seconds": res.compile_ms * 1e-3,
    }
    print(json.dumps(summary), flush=True)
    if a.save:
        b.sgemm_cache_save(a.save)
    return 0


if __name__ == "__main__":
    sys.exit(main())
