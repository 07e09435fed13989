"""Search strategies on synthetic cost tables (no GPU).

First the oracle (oracle/search_oracle.py) is pinned to what the paper and the mathematics
fix: the annealing acceptance formula, limiting cases of both heuristics, published output of
the SplitMix64 generator.  Then the library's strategies (tune_replay through the C ABI) must
reproduce the oracle's searches step by step on the same cost tables and seeds."""
import math

import numpy as np
import pytest

from oracle import search_oracle as so
from oracle import space_oracle as sp
from paper_1703_06503_amd import binding as b


def synthetic_costs(configs, seed, fail_fraction=0.03):
    """A rugged but structured cost surface: product of per-parameter factors times noise,
    with a few failed configurations."""
    rng = np.random.default_rng(seed)
    factors = []
    for d in range(13):
        vals = sorted({c[d] for c in configs})
        factors.append({v: float(f) for v, f in zip(vals, rng.uniform(0.6, 1.8, len(vals)))})
    t = np.array([math.prod(factors[d][c[d]] for d in range(13)) for c in configs])
    t *= rng.uniform(0.9, 1.1, len(configs))
    t[rng.random(len(configs)) < fail_fraction] = -1.0
    return t.astype(np.float32)


SPACES = {p: sp.enumerate_space(p) for p in (sp.SPACE_SMALL, sp.SPACE_FULL)}


# ---------------------------------------------------------------- oracle pins

def test_splitmix64_published_sequence():
    # first outputs for seed 1234567, as published with the reference implementation
    rng = so.SplitMix64(1234567)
    assert [rng.next() for _ in range(5)] == [6457827717110365317, 3203168211198807973,
                                              9817491932198370423, 4593380528125082431,
                                              16408922859458223821]


def test_acceptance_probability_closed_forms():
    # the paper's formula: P = 1 when t' < t, else exp(-(t'-t)/T)
    assert so.acceptance_probability(5.0, 4.0, 2.0) == 1.0
    assert so.acceptance_probability(3.0, 3.0 + 2.0, 2.0) == pytest.approx(math.exp(-1))
    assert so.acceptance_probability(3.0, 3.0, 7.0) == 1.0               # equal times: e^0
    assert so.acceptance_probability(1.0, 13.0, 4.0) == pytest.approx(math.exp(-3))
    # larger T accepts more, larger gap accepts less
    assert so.acceptance_probability(1, 2, 6) > so.acceptance_probability(1, 2, 2)
    assert so.acceptance_probability(1, 3, 4) < so.acceptance_probability(1, 2, 4)


def test_full_search_is_the_argmin():
    cfgs = SPACES[sp.SPACE_SMALL]
    t = synthetic_costs(cfgs, 1, fail_fraction=0.2)
    r = so.full_search(cfgs, t)
    ok = np.where(t > 0, t, np.inf)
    assert r["best_index"] == int(np.argmin(ok)) and r["evaluations"] == len(cfgs)
    assert r["failed"] == int((t <= 0).sum()) and r["visited"] == list(range(len(cfgs)))


def test_random_search_samples_without_replacement_and_fraction_one_is_full():
    cfgs = SPACES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 2)
    r = so.random_search(cfgs, t, 107, seed=5)
    assert len(r["visited"]) == 107 == len(set(r["visited"]))
    small = SPACES[sp.SPACE_SMALL]
    ts = synthetic_costs(small, 3)
    r = so.random_search(small, ts, 0, seed=5, fraction=1.0)
    assert sorted(r["visited"]) == list(range(16))
    assert r["best_index"] == so.full_search(small, ts)["best_index"]
    # a fraction is rounded down to whole configurations, but at least one is explored
    assert so.random_search(small, ts, 0, seed=5, fraction=1 / 32)["evaluations"] == 1
    assert so.random_search(small, ts, 0, seed=5, fraction=3.9 / 16)["evaluations"] == 3
    # uniformity: every configuration is equally likely to be the first pick
    first = np.bincount([so.random_search(small, ts, 1, seed=s)["visited"][0] for s in range(3200)],
                        minlength=16)
    chi2 = float(((first - 200.0) ** 2 / 200.0).sum())
    assert chi2 < 45.0          # 15 degrees of freedom, far tail


def test_budget_from_a_fraction_matches_the_numbers_the_paper_prints():
    """tests/golden/paper_search_budgets.txt: 1/32 of 3424 -> 107, 1/2048 of 241 600 -> 117."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_search_budgets.txt")
    rows = [tuple(int(x) for x in line.split()) for line in open(path)
            if line.strip() and not line.startswith("#")]
    assert rows == [(3424, 32, 107), (241600, 2048, 117)]
    for n, denom, explored in rows:
        configs = [(i,) for i in range(n)]
        t = np.ones(n, dtype=np.float32)
        r = so.random_search(configs, t, 0, seed=1, fraction=1.0 / denom)
        assert r["evaluations"] == explored and len(set(r["visited"])) == explored
    # the library rounds the same way on its own spaces
    n = b.sgemm_space_size(b.SPACE_FULL)
    t = np.ones(n, dtype=np.float32)
    ev, _, visited = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_RANDOM, 0, 1, _opts(random_fraction=1 / 2048))
    assert ev == n // 2048 == len(visited)


def test_annealing_limits():
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 4, fail_fraction=0.0)
    # T -> 0: a worse neighbour is never accepted, so the current state's cost never rises
    r = so.simulated_annealing(cfgs, vals, t, 150, seed=9, T=1e-12)
    cur = [t[s] for s in r["trace"]]
    assert all(b_ <= a_ for a_, b_ in zip(cur, cur[1:]))
    # huge T: nearly every proposal is accepted (a random walk)
    r = so.simulated_annealing(cfgs, vals, t, 150, seed=9, T=1e12)
    moved = sum(a_ != b_ for a_, b_ in zip(r["trace"], r["trace"][1:]))
    assert moved >= 0.9 * (len(r["trace"]) - 1)
    # every step is to a neighbour: exactly one parameter differs
    for a_, b_ in zip(r["trace"], r["trace"][1:]):
        assert sum(x != y for x, y in zip(cfgs[a_], cfgs[b_])) <= 1
    # budget counts distinct configurations and is never exceeded
    assert r["evaluations"] == len(set(r["visited"])) <= 150
    # deterministic per seed, different across seeds
    again = so.simulated_annealing(cfgs, vals, t, 150, seed=9, T=1e12)
    assert again["visited"] == r["visited"]
    assert so.simulated_annealing(cfgs, vals, t, 150, seed=10, T=1e12)["visited"] != r["visited"]


def test_annealing_acceptance_frequency_matches_formula():
    """Two-level cost surface: the start is the best (1.0) and every other configuration is
    4 % slower, so the first proposal has delta = 4 percent and, with T = 4 barely cooled
    (2 of 400 evaluations spent), must be accepted with probability exp(-4 / 3.98)."""
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    n = len(cfgs)
    accepted = tried = 0
    for seed in range(250):
        start = so.SplitMix64(seed).below(n)
        t = np.full(n, 1.04, dtype=np.float32)
        t[start] = 1.0
        r = so.simulated_annealing(cfgs, vals, t, 400, seed=seed, T=4.0)
        assert r["trace"][0] == start
        tried += 1
        accepted += r["trace"][1] != r["trace"][0]
    p_expect = math.exp(-(100.0 * (float(np.float32(1.04)) - 1.0)) / (4.0 * (1 - 2 / 400)))
    p = accepted / tried
    assert abs(p - p_expect) < 4 * math.sqrt(p_expect * (1 - p_expect) / tried)


def test_pso_limits():
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 6, fail_fraction=0.0)
    # (alpha, beta, gamma) = (0, 0, 1): every particle lands on the swarm's best in one step
    r = so.particle_swarm(cfgs, vals, t, 50, seed=3, S=6, alpha=0.0, beta=0.0, gamma=1.0)
    init = [pos for _, pos in r["positions"][:6]]
    g = min(init, key=lambda i: t[i])
    assert all(pos == g for _, pos in r["positions"][6:12])
    # (0, 0, 0): particles never move
    r = so.particle_swarm(cfgs, vals, t, 50, seed=3, S=6, alpha=0.0, beta=0.0, gamma=0.0)
    for i, pos in r["positions"][6:]:
        assert pos == init[i]
    assert r["evaluations"] == len(set(init))
    # (0, 1, 0): a particle returns to its own best, which after the start is where it stands
    r = so.particle_swarm(cfgs, vals, t, 50, seed=3, S=6, alpha=0.0, beta=1.0, gamma=0.0)
    for i, pos in r["positions"][6:]:
        assert pos == init[i]
    # (1, 0, 0): pure random proposals: positions are unrelated to the start and all valid
    r = so.particle_swarm(cfgs, vals, t, 200, seed=3, S=3, alpha=1.0, beta=0.0, gamma=0.0)
    assert r["evaluations"] == 200 and len(set(r["visited"])) == 200
    assert all(0 <= pos < len(cfgs) for _, pos in r["positions"])


def test_pso_per_dimension_frequencies():
    """Paper's update rule with (alpha, beta, gamma) = (0.4, 0, 0.4): in a dimension where the
    particle differs from the swarm's best, the new value equals g_d with probability
    gamma + alpha/|values| and stays x_d with probability (1-alpha-beta-gamma) + alpha/|values|.
    Measured on a space without constraints, where no proposal is ever redrawn."""
    import itertools
    values = tuple([0, 1, 2, 3] if d < 5 else [0] for d in range(13))
    cfgs = list(itertools.product(*values))
    n = len(cfgs)
    to_g = stay = total = 0
    for seed in range(1500):
        rng = so.SplitMix64(seed)
        x0, g = rng.below(n), rng.below(n)       # start of particle 0 and of particle 1
        if x0 == g:
            continue
        t = np.full(n, 2.0, dtype=np.float32)
        t[g] = 1.0                               # particle 1 holds the swarm's best
        r = so.particle_swarm(cfgs, values, t, 3, seed=seed, S=2, alpha=0.4, beta=0.0, gamma=0.4)
        assert r["positions"][0] == (0, x0) and r["positions"][1] == (1, g)
        if len(r["positions"]) < 3:
            continue                              # the move was a revisit ending the budget
        who, new = r["positions"][2]
        assert who == 0
        for d in range(5):
            if cfgs[x0][d] != cfgs[g][d]:
                total += 1
                to_g += cfgs[new][d] == cfgs[g][d]
                stay += cfgs[new][d] == cfgs[x0][d]
    assert total > 3000
    for count, expect in ((to_g, 0.4 + 0.4 / 4), (stay, 0.2 + 0.4 / 4)):
        assert abs(count / total - expect) < 5 * math.sqrt(expect * (1 - expect) / total)


def test_pso_budget_validity_determinism():
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 7)
    r = so.particle_swarm(cfgs, vals, t, 117, seed=11, S=3)
    assert r["evaluations"] == 117 == len(set(r["visited"]))
    assert r["best_cost"] == min(float(t[i]) for i in r["visited"] if t[i] > 0)
    assert so.particle_swarm(cfgs, vals, t, 117, seed=11, S=3)["visited"] == r["visited"]
    assert so.particle_swarm(cfgs, vals, t, 117, seed=12, S=3)["visited"] != r["visited"]


def test_heuristics_beat_random_on_a_structured_surface():
    """The paper's qualitative finding for GEMM: annealing and PSO outperform random search
    at equal budgets.  On a separable surface (where a good value in one parameter is good
    everywhere) both must win on average over many seeds."""
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 8, fail_fraction=0.0)
    budget = 117
    rnd = np.mean([so.random_search(cfgs, t, budget, s)["best_cost"] for s in range(40)])
    sa = np.mean([so.simulated_annealing(cfgs, vals, t, budget, s, T=4.0)["best_cost"] for s in range(40)])
    pso = np.mean([so.particle_swarm(cfgs, vals, t, budget, s, S=3)["best_cost"] for s in range(40)])
    assert sa < rnd and pso < rnd


# ---------------------------------------------------------------- library against the oracle

def _opts(**kw):
    o = b.tune_opts()
    for k, v in kw.items():
        setattr(o, k, v)
    return o


@pytest.mark.parametrize("preset,lib_space", [(sp.SPACE_SMALL, b.SPACE_SMALL), (sp.SPACE_FULL, b.SPACE_FULL)])
def test_library_full_and_random_match_oracle(preset, lib_space):
    cfgs = SPACES[preset]
    t = synthetic_costs(cfgs, 20 + preset, fail_fraction=0.1)
    ev, res, visited = b.tune_replay(lib_space, t, b.STRATEGY_FULL, 0, 0)
    want = so.full_search(cfgs, t)
    assert (ev, res.best_index, res.failed, visited) == (want["evaluations"], want["best_index"],
                                                         want["failed"], want["visited"])
    assert res.best.as_tuple() == cfgs[want["best_index"]] and res.space_size == len(cfgs)
    for seed in (0, 1, 99):
        budget = max(1, len(cfgs) // 8)
        ev, res, visited = b.tune_replay(lib_space, t, b.STRATEGY_RANDOM, budget, seed)
        want = so.random_search(cfgs, t, budget, seed)
        assert visited == want["visited"] and res.best_index == want["best_index"]
        assert res.evals_to_best == want["evals_to_best"]
    ev, res, visited = b.tune_replay(lib_space, t, b.STRATEGY_RANDOM, 0, 4, _opts(random_fraction=1 / 32))
    assert visited == so.random_search(cfgs, t, 0, 4, fraction=1 / 32)["visited"]


@pytest.mark.parametrize("T", [2.0, 4.0, 6.0])
@pytest.mark.parametrize("raw", [0, 1])
def test_library_annealing_matches_oracle(T, raw):
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    for seed in (0, 7):
        t = synthetic_costs(cfgs, 30 + seed)
        ev, res, visited = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_ANNEALING, 117, seed,
                                         _opts(sa_T=T, sa_raw_ms=raw))
        want = so.simulated_annealing(cfgs, vals, t, 117, seed, T=T, raw_ms=bool(raw))
        assert visited == want["visited"]
        assert (res.best_index, ev, res.failed) == (want["best_index"], want["evaluations"], want["failed"])
        assert res.best_ms == pytest.approx(want["best_cost"])


@pytest.mark.parametrize("S", [3, 6])
def test_library_pso_matches_oracle(S):
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    for seed, (al, be, ga) in [(0, (0.4, 0.0, 0.4)), (5, (0.4, 0.0, 0.4)), (6, (0.2, 0.3, 0.3))]:
        t = synthetic_costs(cfgs, 40 + seed)
        ev, res, visited = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_PSO, 117, seed,
                                         _opts(pso_S=S, pso_alpha=al, pso_beta=be, pso_gamma=ga))
        want = so.particle_swarm(cfgs, vals, t, 117, seed, S=S, alpha=al, beta=be, gamma=ga)
        assert visited == want["visited"]
        assert (res.best_index, ev, res.evals_to_best) == (want["best_index"], want["evaluations"],
                                                           want["evals_to_best"])


def test_library_warm_start_matches_oracle():
    """A search continued from a given configuration: annealing starts there, the swarm's
    particle 0 starts there, and no random draw is spent on that start."""
    cfgs = SPACES[sp.SPACE_FULL]
    vals = sp.VALUES[sp.SPACE_FULL]
    t = synthetic_costs(cfgs, 60)
    for start in (0, 1234, len(cfgs) - 1):
        ev, res, visited = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_ANNEALING, 60, 3,
                                         _opts(warm_start=-(start + 1)))
        want = so.simulated_annealing(cfgs, vals, t, 60, 3, start=start)
        assert visited[0] == start and visited == want["visited"]
        ev, res, visited = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_PSO, 60, 3,
                                         _opts(pso_S=3, warm_start=-(start + 1)))
        want = so.particle_swarm(cfgs, vals, t, 60, 3, S=3, start=start)
        assert visited[0] == start and visited == want["visited"]
    # a start that is the optimum is never lost
    tt = np.asarray(t, dtype=np.float64)
    best = int(np.argmin(np.where(np.isfinite(tt) & (tt > 0), tt, np.inf)))
    _, res, _ = b.tune_replay(b.SPACE_FULL, t, b.STRATEGY_ANNEALING, 40, 9, _opts(warm_start=-(best + 1)))
    assert res.best_index == best


def test_library_small_space_all_strategies_and_edge_budgets():
    cfgs = SPACES[sp.SPACE_SMALL]
    vals = sp.VALUES[sp.SPACE_SMALL]
    t = synthetic_costs(cfgs, 50, fail_fraction=0.0)
    for budget in (1, 2, 16, 1000):
        for seed in (0, 3):
            _, _, v = b.tune_replay(b.SPACE_SMALL, t, b.STRATEGY_ANNEALING, budget, seed)
            assert v == so.simulated_annealing(cfgs, vals, t, budget, seed)["visited"]
            _, _, v = b.tune_replay(b.SPACE_SMALL, t, b.STRATEGY_PSO, budget, seed)
            assert v == so.particle_swarm(cfgs, vals, t, budget, seed)["visited"]
            assert len(v) <= min(budget, 16)
    # all configurations failed: no best, an error status, nothing crashes
    dead = np.full(16, -1.0, dtype=np.float32)
    ev, res, _ = b.tune_replay(b.SPACE_SMALL, dead, b.STRATEGY_PSO, 8, 0)
    assert res.best_index == -1 and res.failed == ev
    # wrong table length / unknown strategy
    with pytest.raises(b.SgemmError):
        b.tune_replay(b.SPACE_SMALL, t[:5], b.STRATEGY_FULL, 0, 0)
    with pytest.raises(b.SgemmError):
        b.tune_replay(b.SPACE_SMALL, t, 9, 0, 0)
