#include "space.h"

#include <algorithm>
#include <cstdlib>
#include <mutex>

namespace sgemm {

static const char *kNames[kDims] = {"MWG", "NWG", "KWG", "MDIMC", "NDIMC", "VWM", "VWN",
                                    "SA",  "SB",  "PAD", "KWI",   "MFMA",  "GRP",   "SK",  "NS", "KSW"};

const char *dim_name(int d) { return (d >= 0 && d < kDims) ? kNames[d] : "?"; }

Point to_point(const sgemm_config &c) {
    return Point{c.mwg, c.nwg, c.kwg, c.mdimc, c.ndimc, c.vwm, c.vwn,
                 c.sa,  c.sb,  c.pad, c.kwi,   c.mfma,  c.grp, c.sk > 0 ? c.sk : 1, c.ns > 0 ? c.ns : 2,
                 c.ksw > 0 ? c.ksw : 1};
}

sgemm_config from_point(const Point &p) {
    sgemm_config c{};
    c.mwg = p[0]; c.nwg = p[1]; c.kwg = p[2]; c.mdimc = p[3]; c.ndimc = p[4];
    c.vwm = p[5]; c.vwn = p[6]; c.sa = p[7]; c.sb = p[8]; c.pad = p[9];
    c.kwi = p[10]; c.mfma = p[11]; c.grp = p[12]; c.sk = p[13]; c.ns = p[14]; c.ksw = p[15];
    return c;
}

int threads_of(const sgemm_config &c) { return c.mdimc * c.ndimc * (c.ksw > 1 ? c.ksw : 1); }

int lds_bytes(const sgemm_config &c, int layout) {
    // only register-staged tiles can be padded; LDS-direct tiles are dense
    const int pad_a = (c.pad && c.sa == 1) ? 4 : 0, pad_b = (c.pad && c.sb == 1) ? 4 : 0;
    int words = 0;
    if (c.sa) words += (layout & 1) ? c.kwg * (c.mwg + pad_a) : c.mwg * (c.kwg + pad_a);
    if (c.sb) words += (layout & 2) ? c.nwg * (c.kwg + pad_b) : c.kwg * (c.nwg + pad_b);
    words *= (c.ns > 0 ? c.ns : 2); // ns buffers
    // wave groups hand their sums over through the same memory, one tile of C at a time
    if (c.ksw > 1 && c.mwg * c.nwg > words) words = c.mwg * c.nwg;
    return 4 * words;
}

int lds_bytes(const sgemm_config &c) {
    int worst = 0;
    for (int layout = 0; layout < 4; ++layout) {
        const int b = lds_bytes(c, layout);
        if (b > worst) worst = b;
    }
    return worst;
}

static bool is_pow2_between(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

// Tile edges are 2^a, 3 * 2^a, 5 * 2^a or 7 * 2^a: the odd factors (96, 192; 80, 160; 112, 224)
// let the tile grid fit sizes that powers of two quantise badly (3000 = 15.6 x 192,
// 1536 = 16 x 96, 2560 = 16 x 160, 3584 = 16 x 224).
static bool is_tile_edge(int v, int lo, int hi) {
    if (v < lo || v > hi) return false;
    for (int f : {1, 3, 5, 7})
        if (v % f == 0 && ((v / f) & (v / f - 1)) == 0) return true;
    return false;
}

// Registers a lane needs beside its accumulators: two KWI blocks of operand fragments (the one
// being multiplied and the one fetched ahead), the global->LDS staging registers, two address
// registers per global load instruction of a slab, and 24 for loop state and the epilogue.
int estimated_registers(const sgemm_config &c) {
    const int nt = threads_of(c);
    const int mwi = c.mwg / c.mdimc, nwi = c.nwg / c.ndimc;
    int fragments;
    if (c.mfma) {
        const int mt = c.mfma == 1 ? 32 : 16, mk = c.mfma == 1 ? 2 : 4;
        fragments = ((8 * mwi) / mt + (8 * nwi) / mt) * (c.kwi / mk);
    } else {
        fragments = mwi + nwi;
    }
    int regs = 2 * fragments + 24;
    if (c.sa) regs += 2 * (c.mwg * c.kwg / (nt * c.vwm)) + (c.sa == 1 ? c.mwg * c.kwg / nt : 0);
    if (c.sb) regs += 2 * (c.nwg * c.kwg / (nt * c.vwn)) + (c.sb == 1 ? c.nwg * c.kwg / nt : 0);
    return regs;
}

// 512 registers per lane of a SIMD (VGPRs and accumulation VGPRs together), shared by the
// workgroup's waves on that SIMD: nt / 64 waves on 4 SIMDs.
static int register_budget(int nt) { return 512 / ((nt + 255) / 256); }

bool prefetch_of_c_fits(const sgemm_config &c) {
    if (!c.mfma) return false; // the vector-ALU schedule reads C row by row in its epilogue
    const int mwi = c.mwg / c.mdimc, nwi = c.nwg / c.ndimc;
    // the old values wait in architected registers, of which a wave addresses 256 (variants of
    // 64 or 128 threads that pass the test against their whole budget were seen to spill)
    return 2 * mwi * nwi + estimated_registers(c) <= std::min(register_budget(threads_of(c)), 256);
}

int direct_loads_per_slab(const sgemm_config &c) {
    const int nt = threads_of(c);
    int ops = 0;
    if (c.sa == 2) ops += c.mwg * c.kwg / (nt * c.vwm);
    if (c.sb == 2) ops += c.nwg * c.kwg / (nt * c.vwn);
    return ops;
}

const char *violates(const sgemm_config &c) {
    if (const char *why = violates_structure(c)) return why;
    const int nt = threads_of(c);
    const int mwi = c.mwg / c.mdimc, nwi = c.nwg / c.ndimc;
    // device limit: the register file (without the matrix cores there are no accumulation
    // registers, so 256 at most)
    const int budget = c.mfma ? register_budget(nt) : std::min(register_budget(nt), 256);
    if (mwi * nwi + estimated_registers(c) > budget) return "register budget";
    // 16x16x4 tiles that would take all 256 accumulation registers: every such variant spills
    if (c.mfma == 2 && mwi * nwi >= 256) return "accumulators leave no accumulation register free";
    return nullptr;
}

const char *violates_structure(const sgemm_config &c) {
    if (!is_tile_edge(c.mwg, 8, 512) || !is_tile_edge(c.nwg, 8, 512)) return "tile size";
    if (!is_pow2_between(c.kwg, 2, 128)) return "KWG";
    if (!is_pow2_between(c.mdimc, 1, 64) || !is_pow2_between(c.ndimc, 1, 64)) return "workgroup shape";
    if (c.vwm != 1 && c.vwm != 2 && c.vwm != 4) return "VWM";
    if (c.vwn != 1 && c.vwn != 2 && c.vwn != 4) return "VWN";
    if ((c.pad | c.grp) & ~1) return "flag not 0/1";
    if (c.sa < 0 || c.sa > 2 || c.sb < 0 || c.sb > 2) return "SA/SB";
    if (c.ns != 0 && (c.ns < 2 || c.ns > 4)) return "NS"; // 0 is read as 2
    if (c.mfma < 0 || c.mfma > 2) return "MFMA";
    if (!is_pow2_between(c.kwi, 1, 32)) return "KWI";
    if (c.sk < 0 || c.sk > kMaxSplitK) return "SK"; // 0 is read as 1
    if (c.ksw != 0 && c.ksw != 1 && c.ksw != 2 && c.ksw != 4) return "KSW"; // 0 is read as 1
    if (c.ksw > 1 && !c.mfma) return "KSW > 1 without the matrix-core schedule";
    const int ksw = c.ksw > 1 ? c.ksw : 1;
    const int nt = threads_of(c);
    // device limit: whole wavefronts, at most 1024 threads
    if ((c.mdimc * c.ndimc) % 64 != 0 || nt > kMaxThreads) return "threads per workgroup";
    if (c.mwg % c.mdimc || c.nwg % c.ndimc) return "tile not divisible by workgroup shape";
    const int mwi = c.mwg / c.mdimc, nwi = c.nwg / c.ndimc;
    if (c.kwg % (c.kwi * ksw)) return "KWG not divisible by KWI (times KSW)";
    if (c.sa) {
        if (c.mwg % c.vwm || c.kwg % c.vwm) return "A tile row not divisible by VWM";
        if ((c.mwg * c.kwg) % (nt * c.vwm)) return "A tile not divisible among threads";
    } else if (c.vwm != 1) {
        return "VWM without staging A"; // the width would change nothing: keep one spelling
    }
    if (c.sb) {
        if (c.nwg % c.vwn || c.kwg % c.vwn) return "B tile row not divisible by VWN";
        if ((c.nwg * c.kwg) % (nt * c.vwn)) return "B tile not divisible among threads";
    }
    if (c.pad && c.sa != 1 && c.sb != 1) return "PAD without a register-staged tile";
    // LDS-direct loads move 4 or 16 bytes per lane
    if ((c.sa == 2 && c.vwm == 2) || (c.sb == 2 && c.vwn == 2)) return "LDS-direct load width";
    // a wave counts at most kMaxLoadsInFlight outstanding loads: one slab's LDS-direct loads,
    // and with more than two buffers those of the ns - 2 youngest slabs, must fit
    if (direct_loads_per_slab(c) > kMaxLoadsInFlight) return "loads in flight";
    if (c.ns > 2) {
        if (c.sa == 1 || c.sb == 1 || (c.sa != 2 && c.sb != 2)) return "NS > 2 without LDS-direct staging";
        if ((c.ns - 2) * direct_loads_per_slab(c) > kMaxLoadsInFlight) return "loads in flight";
    }
    if (c.mfma == 0) {
        if (nwi % c.vwn) return "NWI not divisible by VWN";
        if (mwi * nwi > 64) return "register tile too large";
    } else {
        if (c.mdimc % 8 || c.ndimc % 8) return "workgroup shape not made of 8x8 wave patches";
        if (!c.sb && c.vwn != 1) return "VWN without staging B";
        const int mt = c.mfma == 1 ? 32 : 16, mk = c.mfma == 1 ? 2 : 4;
        if ((8 * mwi) % mt || (8 * nwi) % mt) return "wave tile not a multiple of the MFMA tile";
        if (c.kwi % mk) return "KWI not a multiple of the MFMA depth";
        if (mwi * nwi > 256) return "accumulator tile too large";
    }
    // device limit: 160 KiB LDS per workgroup
    if (lds_bytes(c) > kLdsLimitBytes) return "LDS capacity";
    return nullptr;
}

uint64_t Space::key(const Point &p) {
    uint64_t h = 1469598103934665603ull;
    for (int v : p) { h ^= (uint64_t)(uint32_t)v; h *= 1099511628211ull; }
    return h;
}

int Space::find(const Point &p) const {
    auto it = index.find(key(p));
    if (it == index.end()) return -1;
    return configs[it->second] == p ? it->second : -1;
}

static Space build(int preset) {
    Space s;
    s.preset = preset;
    switch (preset) {
    case SGEMM_SPACE_SMALL:
        // MWG, NWG in {32,64}; KWG in {8,16}; staging on/off for both operands together
        s.values = {{32, 64}, {32, 64}, {8, 16}, {8}, {8}, {1}, {1}, {0, 1}, {0, 1}, {0}, {2}, {0}, {0}, {1}, {2}, {1}};
        break;
    case SGEMM_SPACE_FULL:
        s.values = {{32, 64, 128, 256}, {32, 64, 128, 256}, {8, 16, 32}, {8, 16}, {8, 16},
                    {1, 4}, {1, 4}, {0, 1}, {0, 1}, {0, 1}, {2, 8}, {0, 1}, {0, 1}, {1}, {2}, {1}};
        break;
    case SGEMM_SPACE_MFMA:
        s.values = {{64, 128, 256}, {64, 128, 256}, {8, 16, 32}, {8, 16, 32}, {8, 16, 32},
                    {1, 2, 4}, {1, 2, 4}, {1}, {1}, {0, 1}, {2, 8}, {1, 2}, {0, 1}, {1}, {2}, {1}};
        break;
    case SGEMM_SPACE_EXT:
        // matrix-core variants with tile edges 3 * 2^a as well, deeper K slabs, and split K
        s.values = {{32, 64, 96, 128, 192, 256}, {32, 64, 96, 128, 192, 256}, {16, 32, 64},
                    {8, 16, 32}, {8, 16, 32}, {1, 2, 4}, {1, 2, 4}, {1}, {1}, {0, 1}, {2, 8},
                    {1, 2}, {0, 1}, {1, 2, 3, 4, 6, 8, 12, 16}, {2}, {1}};
        break;
    case SGEMM_SPACE_DIRECT:
        // matrix-core variants fed by LDS-direct loads, 2 to 4 LDS buffers per tile
        s.values = {{32, 64, 96, 128, 192, 256}, {32, 64, 96, 128, 192, 256}, {16, 32, 64},
                    {8, 16, 32}, {8, 16, 32}, {1, 4}, {1, 4}, {2}, {2}, {0}, {2, 8},
                    {1, 2}, {0, 1}, {1, 2, 3, 4, 6, 8, 12, 16}, {2, 3, 4}, {1}};
        break;
    case SGEMM_SPACE_KSPLIT:
        // matrix-core variants whose waves share out the K slab: small tiles, 2 or 4 wave groups
        s.values = {{32, 64, 96, 128}, {32, 64, 96, 128}, {32, 64}, {8, 16}, {8, 16}, {4}, {4}, {1}, {1},
                    {0, 1}, {2, 8}, {1, 2}, {0, 1}, {1, 2, 4}, {2}, {2, 4}};
        break;
    default:
        s.preset = -1;
        return s;
    }
    s.raw = 1;
    for (auto &v : s.values) s.raw *= (long long)v.size();
    Point p{};
    std::array<size_t, kDims> it{};
    bool done = false;
    while (!done) {
        for (int d = 0; d < kDims; ++d) p[d] = s.values[d][it[d]];
        sgemm_config c = from_point(p);
        bool ok = violates(c) == nullptr;
        if (preset == SGEMM_SPACE_SMALL && c.sa != c.sb) ok = false; // one LDS switch
        if (ok) {
            s.index.emplace(Space::key(p), (int)s.configs.size());
            s.configs.push_back(p);
        }
        int d = kDims - 1; // odometer, last dimension fastest => lexicographic order
        while (d >= 0 && ++it[d] == s.values[d].size()) { it[d] = 0; --d; }
        if (d < 0) done = true;
    }
    return s;
}

// ---- the caller-defined space ---------------------------------------------------------------
// "NAME=v,v,... NAME=v ..." (names as in dim_name(), separated by blanks or ';'); a parameter
// that is not named keeps the single value given as its default here.
static const int kCustomDefaults[kDims] = {128, 128, 32, 16, 16, 4, 4, 1, 1, 1, 8, 1, 0, 1, 2, 1};

static bool parse_custom(const std::string &spec, std::vector<std::vector<int>> *values) {
    values->assign(kDims, {});
    size_t pos = 0;
    while (pos < spec.size()) {
        while (pos < spec.size() && (spec[pos] == ' ' || spec[pos] == ';' || spec[pos] == '\n' || spec[pos] == '\t')) ++pos;
        if (pos >= spec.size()) break;
        const size_t eq = spec.find('=', pos);
        if (eq == std::string::npos) return false;
        const std::string name = spec.substr(pos, eq - pos);
        int dim = -1;
        for (int d = 0; d < kDims; ++d)
            if (name == kNames[d]) dim = d;
        if (dim < 0 || !(*values)[dim].empty()) return false; // unknown or repeated name
        pos = eq + 1;
        for (;;) {
            size_t end = pos;
            while (end < spec.size() && spec[end] >= '0' && spec[end] <= '9') ++end;
            if (end == pos || end - pos > 6) return false;
            (*values)[dim].push_back(std::atoi(spec.substr(pos, end - pos).c_str()));
            pos = end;
            if (pos < spec.size() && spec[pos] == ',') { ++pos; continue; }
            break;
        }
    }
    for (int d = 0; d < kDims; ++d)
        if ((*values)[d].empty()) (*values)[d].push_back(kCustomDefaults[d]);
    return true;
}

static Space enumerate_values(int preset, std::vector<std::vector<int>> values) {
    Space s;
    s.preset = preset;
    s.values = std::move(values);
    s.raw = 1;
    for (auto &v : s.values) s.raw *= (long long)v.size();
    Point p{};
    std::array<size_t, kDims> it{};
    bool done = false;
    while (!done) {
        for (int d = 0; d < kDims; ++d) p[d] = s.values[d][it[d]];
        if (violates(from_point(p)) == nullptr) {
            s.index.emplace(Space::key(p), (int)s.configs.size());
            s.configs.push_back(p);
        }
        int d = kDims - 1;
        while (d >= 0 && ++it[d] == s.values[d].size()) { it[d] = 0; --d; }
        if (d < 0) done = true;
    }
    return s;
}

static std::mutex g_space_mu;
static std::unordered_map<int, Space *> g_built;

int define_custom_space(const char *spec) {
    std::vector<std::vector<int>> values;
    if (!spec || !parse_custom(spec, &values)) return -1;
    long long raw = 1;
    for (auto &v : values) {
        raw *= (long long)v.size();
        if (raw > 50000000ll) return -1; // enumeration is a plain walk of the product
    }
    Space *fresh = new Space(enumerate_values(SGEMM_SPACE_CUSTOM, std::move(values)));
    std::lock_guard<std::mutex> lock(g_space_mu);
    // an earlier definition is kept alive: searches still running may hold a pointer to it
    g_built[SGEMM_SPACE_CUSTOM] = fresh;
    return (int)fresh->configs.size();
}

const Space *get_space(int preset) {
    {
        std::lock_guard<std::mutex> lock(g_space_mu);
        auto it = g_built.find(preset);
        if (it != g_built.end()) return it->second;
    }
    if (preset == SGEMM_SPACE_CUSTOM) {
        // not defined by a call: the environment may define it (worker processes that compile a
        // space in parallel learn it this way)
        const char *env = std::getenv("SGEMM_TUNED_CUSTOM_SPACE");
        if (!env || define_custom_space(env) < 0) return nullptr;
        std::lock_guard<std::mutex> lock(g_space_mu);
        return g_built[SGEMM_SPACE_CUSTOM];
    }
    Space s = build(preset);
    if (s.preset < 0) return nullptr;
    Space *keep = new Space(std::move(s));
    std::lock_guard<std::mutex> lock(g_space_mu);
    auto ins = g_built.emplace(preset, keep);
    if (!ins.second) delete keep;
    return ins.first->second;
}

} // namespace sgemm
