"""Replay the search strategies against a recorded full search (no GPU needed).

    python -m paper_1703_06503_amd.strategy_study results/full_search_cfg2_2048.csv \\
        --space full --budget 500 --runs 128

The table is what `tune_cli --strategy full --log ...` recorded, reduced to `index,ms,status`
(`--from-log` converts a JSONL log).  For each strategy setting of the paper (annealing with
T = 2, 4, 6; particle swarm with S = 3, 6 and (alpha, beta, gamma) = (0.4, 0, 0.4); random
search) the search is repeated with `--runs` seeds, as the paper repeats every search 128
times, and the distribution of the best-found time relative to the full-search optimum is
summarised."""
import argparse
import csv
import json
import sys

import numpy as np

SPACES = {"full": 0, "small": 1, "mfma": 2}
CONV_SPACES = {"conv3x3": (3, 3), "conv7x7": (7, 7), "conv11x11": (11, 11)}  # second kernel family


def space_size_and_replay(name):
    """(number of configurations, replay(table, strategy, budget, seed, opts)) of a named space."""
    from . import binding as b
    if name in CONV_SPACES:
        Xf, Yf = CONV_SPACES[name]
        return (b.conv2d_space_size(Xf, Yf),
                lambda t, strategy, budget, seed, opts: b.conv2d_tune_replay(Xf, Yf, t, strategy, budget, seed, opts))
    space = SPACES[name]
    return (b.sgemm_space_size(space),
            lambda t, strategy, budget, seed, opts: b.tune_replay(space, t, strategy, budget, seed, opts))


def convert_log(jsonl_path, csv_path):
    rows = {}
    with open(jsonl_path) as f:
        for line in f:
            r = json.loads(line)
            rows[r["index"]] = (r["ms"], r["status"])
    with open(csv_path, "w") as f:
        f.write("index,ms,status\n")
        for i in sorted(rows):
            ms, st = rows[i]
            f.write(f"{i},{ms:.6g},{st}\n")
    return len(rows)


def load_table(csv_path, n):
    t = np.full(n, -1.0, dtype=np.float32)
    with open(csv_path) as f:
        for r in csv.DictReader(f):
            if r["status"].startswith("ok"):
                t[int(r["index"])] = float(r["ms"])
    return t


def study(table, space, budget, runs):
    """space: a preset number of the GEMM family, or a replay function of space_size_and_replay()."""
    from . import binding as b
    replay = space if callable(space) else (
        lambda t, strategy, budget, seed, opts: b.tune_replay(space, t, strategy, budget, seed, opts))
    ok = table[table > 0]
    opt = float(ok.min())
    settings = [("random", b.STRATEGY_RANDOM, {})]
    for T in (2.0, 4.0, 6.0):
        settings.append((f"annealing T={T:g}", b.STRATEGY_ANNEALING, {"sa_T": T}))
    for S in (3, 6):
        settings.append((f"pso S={S}", b.STRATEGY_PSO,
                         {"pso_S": S, "pso_alpha": 0.4, "pso_beta": 0.0, "pso_gamma": 0.4}))
    out = []
    for name, strategy, kw in settings:
        opts = b.tune_opts()
        for k, v in kw.items():
            setattr(opts, k, v)
        rel, to5 = [], []
        for seed in range(runs):
            ev, res, visited = replay(table, strategy, budget, seed, opts)
            rel.append(opt / res.best_ms)          # fraction of the optimum's speed reached
            # evaluations spent until a configuration within 5 % of the optimum was timed
            hit = next((i + 1 for i, v in enumerate(visited) if 0 < table[v] <= 1.05 * opt), None)
            to5.append(hit)
        rel = np.array(rel)
        hits = [h for h in to5 if h is not None]
        out.append({
            "strategy": name, "budget": budget, "runs": runs,
            "mean_pct_of_best": 100 * rel.mean(), "median_pct_of_best": 100 * np.median(rel),
            "min_pct_of_best": 100 * rel.min(), "p10_pct_of_best": 100 * np.percentile(rel, 10),
            "runs_within_5pct": int((rel >= 1 / 1.05).sum()),
            "median_evals_to_within_5pct": float(np.median(hits)) if hits else None,
        })
    return opt, out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("table")
    ap.add_argument("--from-log", default=None, help="JSONL log to convert into TABLE first")
    ap.add_argument("--space", choices=sorted(SPACES) + sorted(CONV_SPACES), default="full")
    ap.add_argument("--budget", type=int, nargs="+", default=[500])
    ap.add_argument("--runs", type=int, default=128)
    a = ap.parse_args(argv)
    if a.from_log:
        print(f"converted {convert_log(a.from_log, a.table)} evaluations", file=sys.stderr)
    n, space = space_size_and_replay(a.space)
    table = load_table(a.table, n)
    ok = table[table > 0]
    print(f"space {a.space}: {n} configurations, {len(ok)} with a time, optimum {ok.min():.4f} ms; "
          f"{int((ok <= 1.05 * ok.min()).sum())} within 5 % of it, "
          f"{int((ok <= 1.10 * ok.min()).sum())} within 10 %; mean of the space reaches "
          f"{100 * (ok.min() / ok).mean():.1f} % of the optimum's speed")
    for budget in a.budget:
        opt, rows = study(table, space, budget, a.runs)
        print(f"\nbudget {budget} evaluations ({100 * budget / n:.2f} % of the space), {a.runs} runs each")
        print("| strategy | mean % of best | median | 10th pct | worst | runs within 5 % | median evals to within 5 % |")
        print("|---|---|---|---|---|---|---|")
        for r in rows:
            me = "-" if r["median_evals_to_within_5pct"] is None else f"{r['median_evals_to_within_5pct']:.0f}"
            print(f"| {r['strategy']} | {r['mean_pct_of_best']:.1f} | {r['median_pct_of_best']:.1f} | "
                  f"{r['p10_pct_of_best']:.1f} | {r['min_pct_of_best']:.1f} | "
                  f"{r['runs_within_5pct']}/{r['runs']} | {me} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
