"""Oracle for the four search strategies.  TEST INFRASTRUCTURE ONLY; shares no code with the
library.  Each function takes the algorithm's steps in the paper's order and notation
(sections "Search strategies and search-space properties", "Simulated annealing", "Particle
swarm optimisation") and works on a table of known costs t[i] (milliseconds; a value that is
not a finite positive number marks a failed configuration and counts as +infinity).

Randomness: both this oracle and the library draw from the same public generator, SplitMix64
(Steele, Lea, Flood 2014), so that a search is a function of (space, costs, seed, parameters)
and the two traces can be compared element by element.
    next()    : state += 0x9E3779B97F4A7C15; z = state; z = (z ^ z>>30) * 0xBF58476D1CE4E5B9;
                z = (z ^ z>>27) * 0x94D049BB133111EB; return z ^ z>>31            (mod 2^64)
    below(n)  : next() % n
    uniform() : (next() >> 11) / 2^53

Readings where the paper is silent (the library documents the same ones):
  - budget = number of DISTINCT configurations whose cost is asked for; a revisit is free;
    a search also stops after 20*budget moves.
  - random search: the first `budget` steps of a Fisher-Yates shuffle of 0..n-1.  A budget
    given as a fraction of the space is rounded down (the paper explores 1/2048 of 241 600
    configurations as 117 and 1/32 of 3424 as 107), but is at least 1.
  - annealing: start s = below(n), or a given configuration (then no draw is made: a search
    may be continued from a known good point).  Neighbours of s = valid configurations differing from s
    in exactly one parameter, ordered by parameter then by position in its value list; s' is
    drawn uniformly from them (from the whole space if there are none).  The paper's formula
    has a single T but says the temperature decreases over the search: T_i = T * (1 - e/budget)
    with e = evaluations made so far (including s'), floored at 1e-9.  Execution times are
    compared in percent of the best time found so far (scale-free; raw milliseconds optional):
    P = 1 if t' < t, else exp(-(t' - t) / T_i).  A failed s' is never accepted; a failed s is
    always left.
  - particle swarm: positions start at below(n) for each of the S particles in turn (particle
    0 at the given start configuration, if there is one) and are evaluated; then particles move one at a time, round robin.  For each dimension d one
    uniform() decides: < alpha: epsilon_d = values[d][below(len)], < alpha+beta: p_i,d,
    < alpha+beta+gamma: g_d, else x_i,d.  An invalid mix is redrawn up to 10 times, then the
    particle jumps to below(n).  p_i and g are updated right after every evaluation.
"""
import math

MASK = (1 << 64) - 1


class SplitMix64:
    def __init__(self, seed):
        self.state = seed & MASK

    def next(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
        return z ^ (z >> 31)

    def below(self, n):
        return self.next() % n

    def uniform(self):
        return (self.next() >> 11) / 9007199254740992.0


class _Costs:
    """Budgeted, memoised view of the cost table."""

    def __init__(self, t, budget):
        self.t = t
        self.budget = budget
        self.known = {}
        self.visited = []
        self.best_index = -1
        self.best_cost = math.inf
        self.evals_to_best = 0
        self.failed = 0

    def affordable(self, i):
        return i in self.known or len(self.visited) < self.budget

    def __call__(self, i):
        if i in self.known:
            return self.known[i]
        c = float(self.t[i])
        if not (c > 0.0 and math.isfinite(c)):
            c = math.inf
            self.failed += 1
        self.known[i] = c
        self.visited.append(i)
        if c < self.best_cost:
            self.best_cost, self.best_index, self.evals_to_best = c, i, len(self.visited)
        return c

    def result(self, **extra):
        out = dict(best_index=self.best_index, best_cost=self.best_cost,
                   evaluations=len(self.visited), failed=self.failed,
                   evals_to_best=self.evals_to_best, visited=list(self.visited))
        out.update(extra)
        return out


def acceptance_probability(t, t_new, T):
    """The paper's P(t, t', T)."""
    if t_new < t:
        return 1.0
    return math.exp(-(t_new - t) / T)


def full_search(configs, t):
    costs = _Costs(t, len(configs))
    for i in range(len(configs)):
        costs(i)
    return costs.result()


def random_search(configs, t, budget, seed, fraction=0.0):
    n = len(configs)
    if budget <= 0:
        budget = max(1, math.floor(fraction * n))
    budget = max(1, min(budget, n))
    costs = _Costs(t, budget)
    rng = SplitMix64(seed)
    perm = list(range(n))
    for i in range(budget):
        j = i + rng.below(n - i)
        perm[i], perm[j] = perm[j], perm[i]
        costs(perm[i])
    return costs.result()


def neighbours(configs, values, index_of, s):
    out = []
    for d, vals in enumerate(values):
        for v in vals:
            if v == configs[s][d]:
                continue
            cand = configs[s][:d] + (v,) + configs[s][d + 1:]
            j = index_of.get(cand)
            if j is not None:
                out.append(j)
    return out


def simulated_annealing(configs, values, t, budget, seed, T=4.0, raw_ms=False, start=None):
    n = len(configs)
    budget = max(1, min(budget, n))
    index_of = {c: i for i, c in enumerate(configs)}
    costs = _Costs(t, budget)
    rng = SplitMix64(seed)
    s = rng.below(n) if start is None else start
    t_s = costs(s)
    trace = [s]
    moves = 0
    while moves < 20 * budget and len(costs.visited) < budget:
        moves += 1
        nb = neighbours(configs, values, index_of, s)
        s_new = nb[rng.below(len(nb))] if nb else rng.below(n)
        if not costs.affordable(s_new):
            break
        t_new = costs(s_new)
        T_i = max(T * (1.0 - len(costs.visited) / budget), 1e-9)
        if t_new < t_s or not math.isfinite(t_s):
            accept = True
        elif not math.isfinite(t_new):
            accept = False
        else:
            scale = 1.0 if raw_ms else 100.0 / costs.best_cost
            accept = rng.uniform() < acceptance_probability(t_s * scale, t_new * scale, T_i)
        if accept:
            s, t_s = s_new, t_new
        trace.append(s)
    return costs.result(trace=trace)


def particle_swarm(configs, values, t, budget, seed, S=3, alpha=0.4, beta=0.0, gamma=0.4,
                   start=None):
    n = len(configs)
    budget = max(1, min(budget, n))
    index_of = {c: i for i, c in enumerate(configs)}
    costs = _Costs(t, budget)
    rng = SplitMix64(seed)
    x, p, p_cost = [], [], []
    g, g_cost = -1, math.inf
    positions = []                      # (particle, position) after every move
    for i in range(S):
        xi = start if (i == 0 and start is not None) else rng.below(n)
        if not costs.affordable(xi):
            return costs.result(positions=positions)
        c = costs(xi)
        x.append(xi); p.append(xi); p_cost.append(c)
        if g < 0 or c < g_cost:
            g, g_cost = xi, c
        positions.append((i, xi))
    moves = 0
    while len(costs.visited) < budget and moves < 20 * budget:
        for i in range(S):
            if not (len(costs.visited) < budget and moves < 20 * budget):
                break
            moves += 1
            new = None
            for _ in range(10):
                mix = []
                for d, vals in enumerate(values):
                    u = rng.uniform()
                    if u < alpha:
                        mix.append(vals[rng.below(len(vals))])      # epsilon_d
                    elif u < alpha + beta:
                        mix.append(configs[p[i]][d])                # local best
                    elif u < alpha + beta + gamma:
                        mix.append(configs[g][d])                   # global best
                    else:
                        mix.append(configs[x[i]][d])                # current position
                new = index_of.get(tuple(mix))
                if new is not None:
                    break
            if new is None:
                new = rng.below(n)
            if not costs.affordable(new):
                return costs.result(positions=positions)
            x[i] = new
            c = costs(new)
            positions.append((i, new))
            if c < p_cost[i]:
                p[i], p_cost[i] = new, c
            if c < g_cost:
                g, g_cost = new, c
    return costs.result(positions=positions)
