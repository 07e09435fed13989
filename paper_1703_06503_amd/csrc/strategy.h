// The four search strategies of the tuner over an enumerated space, independent of how a
// configuration's cost is obtained (GPU timing or a recorded table).
// Paper: sections "Search strategies and search-space properties", "Simulated annealing"
// and "Particle swarm optimisation".
#pragma once
#include <cstdint>
#include <functional>
#include <vector>

#include "space.h"

namespace sgemm {

// SplitMix64 sequence: the one source of randomness of every strategy, so that a search is a
// pure function of (space, costs, seed, parameters).
struct Rng {
    uint64_t state;
    explicit Rng(uint64_t seed) : state(seed) {}
    uint64_t next();
    uint64_t below(uint64_t n) { return next() % n; }                   // n > 0
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); } // [0,1)
};

struct StrategyParams {
    double sa_T = 4.0;        // annealing temperature
    bool sa_raw_ms = false;   // false: t'-t measured in percent of the best time so far
    int pso_S = 3;            // swarm size
    double pso_alpha = 0.4, pso_beta = 0.0, pso_gamma = 0.4;
    double random_fraction = 0.0; // random search budget as a fraction when budget <= 0
    int start_index = -1;     // >= 0: annealing starts here, and so does particle 0 of the
                              // swarm, instead of at a random configuration (no draw is made)
};

struct SearchResult {
    int best_index = -1;
    double best_cost = 0.0;
    int evaluations = 0;    // distinct configurations whose cost was asked for
    int failed = 0;         // of those, how many had no valid cost
    int evals_to_best = 0;  // value of `evaluations` when the best was found
    std::vector<int> visited; // distinct configurations in evaluation order
};

// cost(index) -> milliseconds; a non-finite or non-positive value marks a failed configuration.
using CostFn = std::function<double(int)>;

// budget = maximum number of distinct configurations evaluated (full search ignores it).
SearchResult run_search(const Space &space, int strategy, int budget, uint64_t seed,
                        const StrategyParams &params, const CostFn &cost);

// Valid configurations that differ from configs[index] in exactly one parameter, ordered by
// parameter, then by position in that parameter's value list.
std::vector<int> neighbours(const Space &space, int index);

// The annealing acceptance probability of the paper's formula for t' >= t.
double sa_probability(double t, double t_new, double T);

} // namespace sgemm
