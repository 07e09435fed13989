#include "strategy.h"

#include <cmath>
#include <limits>

namespace sgemm {

uint64_t Rng::next() {
    state += 0x9E3779B97F4A7C15ull;
    uint64_t z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

std::vector<int> neighbours(const Space &space, int index) {
    std::vector<int> out;
    const Point &cur = space.configs[index];
    for (int d = 0; d < space.dims; ++d) {
        for (int v : space.values[d]) {
            if (v == cur[d]) continue;
            Point p = cur;
            p[d] = v;
            const int j = space.find(p);
            if (j >= 0) out.push_back(j);
        }
    }
    return out;
}

double sa_probability(double t, double t_new, double T) {
    if (t_new < t) return 1.0;
    return std::exp(-(t_new - t) / T);
}

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

// Memoised, budgeted access to the cost function.
struct Evaluator {
    const CostFn &fn;
    int budget;
    std::vector<double> cost;   // NaN = not evaluated yet; +inf = failed
    SearchResult res;

    Evaluator(const CostFn &f, int n, int b) : fn(f), budget(b), cost(n, std::nan("")) {
        res.best_cost = kInf;
    }
    bool seen(int i) const { return !std::isnan(cost[i]); }
    bool can_afford(int i) const { return seen(i) || res.evaluations < budget; }
    double get(int i) {
        if (seen(i)) return cost[i];
        double c = fn(i);
        if (!(c > 0.0) || !std::isfinite(c)) { c = kInf; ++res.failed; }
        cost[i] = c;
        ++res.evaluations;
        res.visited.push_back(i);
        if (c < res.best_cost) {
            res.best_cost = c;
            res.best_index = i;
            res.evals_to_best = res.evaluations;
        }
        return c;
    }
};

void full_search(Evaluator &ev, int n) {
    for (int i = 0; i < n; ++i) ev.get(i);
}

void random_search(Evaluator &ev, int n, Rng &rng) {
    // sampling without replacement: the first `budget` steps of a Fisher-Yates shuffle
    std::vector<int> perm(n);
    for (int i = 0; i < n; ++i) perm[i] = i;
    for (int i = 0; i < ev.budget && i < n; ++i) {
        const int j = i + (int)rng.below((uint64_t)(n - i));
        std::swap(perm[i], perm[j]);
        ev.get(perm[i]);
    }
}

void annealing(Evaluator &ev, const Space &space, Rng &rng, const StrategyParams &p) {
    const int n = (int)space.configs.size();
    int cur = (p.start_index >= 0 && p.start_index < n) ? p.start_index : (int)rng.below((uint64_t)n);
    double t = ev.get(cur);
    const long long max_steps = 20ll * ev.budget;
    for (long long step = 0; step < max_steps && ev.res.evaluations < ev.budget; ++step) {
        const std::vector<int> nb = neighbours(space, cur);
        const int cand = nb.empty() ? (int)rng.below((uint64_t)n) : nb[rng.below(nb.size())];
        if (!ev.can_afford(cand)) break;
        const double t_new = ev.get(cand);
        // the temperature falls linearly with the share of the budget already spent
        double T = p.sa_T * (1.0 - (double)ev.res.evaluations / (double)ev.budget);
        if (T < 1e-9) T = 1e-9;
        bool accept;
        if (t_new < t || !std::isfinite(t)) {
            accept = true;
        } else if (!std::isfinite(t_new)) {
            accept = false;
        } else {
            const double scale = p.sa_raw_ms ? 1.0 : 100.0 / ev.res.best_cost;
            accept = rng.uniform() < sa_probability(t * scale, t_new * scale, T);
        }
        if (accept) { cur = cand; t = t_new; }
    }
}

void particle_swarm(Evaluator &ev, const Space &space, Rng &rng, const StrategyParams &p) {
    const int n = (int)space.configs.size();
    const int S = p.pso_S > 0 ? p.pso_S : 1;
    std::vector<int> x(S), best(S);
    std::vector<double> best_cost(S);
    int g = -1;
    double g_cost = kInf;
    for (int i = 0; i < S; ++i) {
        x[i] = (i == 0 && p.start_index >= 0 && p.start_index < n) ? p.start_index
                                                                   : (int)rng.below((uint64_t)n);
        if (!ev.can_afford(x[i])) return;
        const double c = ev.get(x[i]);
        best[i] = x[i];
        best_cost[i] = c;
        if (g < 0 || c < g_cost) { g = x[i]; g_cost = c; }
    }
    const long long max_steps = 20ll * ev.budget;
    long long step = 0;
    while (ev.res.evaluations < ev.budget && step < max_steps) {
        for (int i = 0; i < S && ev.res.evaluations < ev.budget && step < max_steps; ++i, ++step) {
            int next = -1;
            for (int attempt = 0; attempt < 10 && next < 0; ++attempt) {
                Point q{}; // entries beyond space.dims stay zero, as in every stored point
                for (int d = 0; d < space.dims; ++d) {
                    const double u = rng.uniform();
                    if (u < p.pso_alpha) {
                        q[d] = space.values[d][rng.below(space.values[d].size())];
                    } else if (u < p.pso_alpha + p.pso_beta) {
                        q[d] = space.configs[best[i]][d];
                    } else if (u < p.pso_alpha + p.pso_beta + p.pso_gamma) {
                        q[d] = space.configs[g][d];
                    } else {
                        q[d] = space.configs[x[i]][d];
                    }
                }
                next = space.find(q);
            }
            if (next < 0) next = (int)rng.below((uint64_t)n); // no valid mix found
            if (!ev.can_afford(next)) return;
            x[i] = next;
            const double c = ev.get(next);
            if (c < best_cost[i]) { best[i] = next; best_cost[i] = c; }
            if (c < g_cost) { g = next; g_cost = c; }
        }
    }
}

} // namespace

SearchResult run_search(const Space &space, int strategy, int budget, uint64_t seed,
                        const StrategyParams &params, const CostFn &cost) {
    const int n = (int)space.configs.size();
    if (n == 0) return SearchResult{};
    int b = budget;
    if (strategy == SGEMM_STRATEGY_FULL) b = n;
    if (strategy == SGEMM_STRATEGY_RANDOM && b <= 0)
        b = (int)std::floor(params.random_fraction * n); // the paper's 1/2048 of 241 600 is 117
    if (b < 1) b = 1;
    if (b > n) b = n;
    Evaluator ev(cost, n, b);
    Rng rng(seed);
    switch (strategy) {
    case SGEMM_STRATEGY_FULL: full_search(ev, n); break;
    case SGEMM_STRATEGY_RANDOM: random_search(ev, n, rng); break;
    case SGEMM_STRATEGY_ANNEALING: annealing(ev, space, rng, params); break;
    case SGEMM_STRATEGY_PSO: particle_swarm(ev, space, rng, params); break;
    default: break;
    }
    return ev.res;
}

} // namespace sgemm
