"""Cross-shape transfer of tuned configurations: run the best configuration found for each
workload on every other workload and print how much of that workload's own best it reaches.

    python -m paper_1703_06503_amd.shape_study --table results/tuned_configs.txt \\
        cfg3_1000 cfg3_1536 cfg3_3000

The paper does this across devices (its GEMM best-parameter table and the 50 % / 61 % / 79 %
figures of the matrix-multiplication case study) and across filter sizes (convolution case
study); with one device the analogue is across problem shapes.  Every timed result is first
compared with the device reference kernel under the library's parity bound."""
import argparse
import statistics
import sys


def time_config(b, torch, cfg, w, dA, dB, dC, dC0, lda, ldb, ldc, reps=11, warm_ms=25.0,
                entry=None):
    """Median milliseconds per call of one configuration on resident operands."""
    run = entry or b.sgemm_run_config

    def call():
        run(None, cfg, w.M, w.N, w.K, w.alpha, dA, lda, dB, ldb, w.beta, dC, ldc,
                           w.layout)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    dC.copy_(dC0)
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


def verified(b, torch, cfg, w, dA, dB, dC, dC0, dRef, lda, ldb, ldc, entry=None):
    dC.copy_(dC0)
    (entry or b.sgemm_run_config)(None, cfg, w.M, w.N, w.K, w.alpha, dA, lda, dB, ldb, w.beta, dC, ldc, w.layout)
    torch.cuda.synchronize()
    bound = 1e-5 * w.K * float(dA.abs().max()) * float(dB.abs().max()) + 1e-6 * dRef.abs()
    return bool(((dC - dRef).abs() <= bound).all())


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("workloads", nargs="+")
    ap.add_argument("--table", required=True, help="best-configuration table (tune_cli --save)")
    a = ap.parse_args(argv)

    import torch
    from . import binding as b
    from . import synth

    b.sgemm_cache_clear()
    b.sgemm_cache_load(a.table)
    ws = [synth.WORKLOADS[n] for n in a.workloads]
    best = {}
    for w in ws:
        cfg = b.sgemm_config_get(w.M, w.N, w.K, w.layout)
        if cfg is None:
            print(f"no tuned configuration for {w.name} in {a.table}", file=sys.stderr)
            return 1
        best[w.name] = cfg
    peak, _, _ = b.sgemm_device_peak()
    ms = {}
    for w in ws:
        A, B, C = synth.make_workload(w)
        dA, dB, dC0 = (torch.from_numpy(x).cuda() for x in (A, B, C))
        dC = dC0.clone()
        dRef = dC0.clone()
        lda, ldb, ldc = A.shape[1], B.shape[1], w.N
        b.sgemm_reference(None, w.M, w.N, w.K, w.alpha, dA, lda, dB, ldb, w.beta, dRef, ldc, w.layout)
        for src in ws:
            cfg = best[src.name]
            if not verified(b, torch, cfg, w, dA, dB, dC, dC0, dRef, lda, ldb, ldc):
                print(f"{src.name}'s configuration fails verification on {w.name}", file=sys.stderr)
                return 1
            ms[w.name, src.name] = time_config(b, torch, cfg, w, dA, dB, dC, dC0, lda, ldb, ldc)
            print(f"# {w.name} with the configuration of {src.name}: {ms[w.name, src.name]:.4f} ms",
                  flush=True)
    print()
    print("Best parameters per shape:")
    print()
    print("| shape | " + " | ".join(n.upper() for n in b.CONFIG_FIELDS) + " |")
    print("|---|" + "---|" * len(b.CONFIG_FIELDS))
    for w in ws:
        print(f"| {w.name} | " + " | ".join(str(v) for v in best[w.name].as_tuple()) + " |")
    print()
    print("GFLOP/s (and % of the row's best) of each shape, run with the configuration tuned "
          "for the column's shape:")
    print()
    print("| run on \\ tuned for | " + " | ".join(w.name for w in ws) + " |")
    print("|---|" + "---|" * len(ws))
    for w in ws:
        flops = 2.0 * w.M * w.N * w.K
        row_best = min(ms[w.name, s.name] for s in ws)
        cells = []
        for s in ws:
            t = ms[w.name, s.name]
            cells.append(f"{flops / t * 1e-6:.0f} ({100.0 * row_best / t:.0f} %)")
        print(f"| {w.name} | " + " | ".join(cells) + " |")
    print()
    print(f"(FP32 peak of this device: {peak:.0f} GFLOP/s)")
    return 0


if __name__ == "__main__":
    sys.exit(main())
