"""Print a best-configuration table (tune_cli --save, or the committed tuned_configs.txt) as
markdown: time, GFLOP/s, fraction of the FP32 peak and algorithmic HBM GB/s per shape.

    python -m paper_1703_06503_amd.report [table] [--peak-tflops 157.3]

Needs no GPU.  GFLOP/s = 2*M*N*K / time; the byte count is A, B read once and C written once
(the table does not record beta, so C is not counted as read)."""
import argparse
import os
import sys

FIELDS = ("MWG", "NWG", "KWG", "MDIMC", "NDIMC", "VWM", "VWN", "SA", "SB", "PAD", "KWI", "MFMA",
          "GRP", "SK", "NS", "KSW")
LAYOUTS = {0: "A M×K, B K×N", 1: "A K×M, B K×N", 2: "A M×K, B N×K", 3: "A K×M, B N×K"}


def read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            if len(p) < 18:
                continue
            M, N, K, layout = (int(x) for x in p[:4])
            ms = float(p[4])
            cfg = [int(x) for x in p[5:]]
            cfg += [1, 2, 1][len(cfg) - 13:]       # SK, NS and KSW columns of older tables
            rows.append((M, N, K, layout, ms, cfg))
    return rows


def main(argv=None):
    here = os.path.dirname(os.path.abspath(__file__))
    ap = argparse.ArgumentParser()
    ap.add_argument("table", nargs="?", default=os.path.join(here, "tuned_configs.txt"))
    ap.add_argument("--peak-tflops", type=float, default=157.3)
    a = ap.parse_args(argv)
    rows = sorted(read_table(a.table), key=lambda r: (r[3], r[0] * r[1] * r[2]))
    print("| M | N | K | storage | ms | GFLOP/s | % of FP32 peak | GB/s (A+B+C once) | "
          + " | ".join(FIELDS) + " |")
    print("|" + "---|" * (8 + len(FIELDS)))
    for M, N, K, layout, ms, cfg in rows:
        flops = 2.0 * M * N * K
        gflops = flops / (ms * 1e-3) * 1e-9
        gbs = 4.0 * (M * K + K * N + M * N) / (ms * 1e-3) * 1e-9
        print(f"| {M} | {N} | {K} | {LAYOUTS[layout]} | {ms:.4f} | {gflops:.0f} | "
              f"{100.0 * gflops / (a.peak_tflops * 1e3):.1f} | {gbs:.0f} | "
              + " | ".join(str(v) for v in cfg) + " |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
