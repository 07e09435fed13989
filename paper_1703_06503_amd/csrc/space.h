// The tuning-parameter space of the SGEMM kernel family: value lists per parameter, the
// constraints that prune their cartesian product, and the enumerated valid configurations.
// (Paper: "Advanced usage" for constraints and device limits; "Tuning parameters" of the
// matrix-multiplication case study for the parameters themselves.)
#pragma once
#include <array>
#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/sgemm_tuned.h"

namespace sgemm {

constexpr int kDims = 16;              // tuned fields of sgemm_config, in field order
constexpr int kLdsLimitBytes = 163840; // LDS per workgroup on gfx950
constexpr int kMaxThreads = 1024;
constexpr int kMaxSplitK = 64;         // upper bound of the SK parameter
// Largest leading dimension of A and B (floats): a tile of up to 512 stored rows then spans
// less than 2 GiB, the reach of the kernels' 32-bit byte offsets and buffer windows.
constexpr int kMaxLeadingDim = 1 << 20;
// M, N, K up to here: rounding a size up to a tile edge (at most 512) stays inside an int
constexpr int kMaxSize = 0x7fffffff - 1024;
constexpr int kMaxLoadsInFlight = 63;  // the vmcnt counter of a wave

using Point = std::array<int, kDims>;

Point to_point(const sgemm_config &c);
sgemm_config from_point(const Point &p);
const char *dim_name(int d);

// Derived quantities of one configuration.
int lds_bytes(const sgemm_config &c);       // worst case over the four storage layouts
int lds_bytes(const sgemm_config &c, int layout);
int estimated_registers(const sgemm_config &c); // beside the accumulators
int direct_loads_per_slab(const sgemm_config &c); // LDS-direct load instructions per thread
// Whether a lane has registers to hold the old values of its part of C beside its accumulators
// (builds for beta != 0 then request them before the first slab instead of in the epilogue).
bool prefetch_of_c_fits(const sgemm_config &c);
int threads_of(const sgemm_config &c);            // mdimc * ndimc * ksw

// nullptr if c satisfies every constraint, else a short reason.
const char *violates(const sgemm_config &c);
// The same without the register-budget rules: what a variant must satisfy to be built and
// launched at all.  (A configuration of a search space passes violates(); the build a call
// really launches may have narrower load vectors than the configuration, hence more load
// instructions and a larger register estimate, and still has to run.)
const char *violates_structure(const sgemm_config &c);

struct Space {
    int preset = -1;
    int dims = kDims;                     // leading entries of a Point that are parameters
    std::vector<std::vector<int>> values; // per dimension
    std::vector<Point> configs;           // valid points, lexicographic in dimension order
    std::unordered_map<uint64_t, int> index;
    long long raw = 0;

    int find(const Point &p) const;
    static uint64_t key(const Point &p);
};

// Built once per preset and kept; nullptr for an unknown preset (or the custom one before it
// has been defined).
const Space *get_space(int preset);

// Defines SGEMM_SPACE_CUSTOM from "NAME=v,v,... NAME=v ..."; returns the number of valid
// configurations, or -1 when the text cannot be read.
int define_custom_space(const char *spec);

} // namespace sgemm
