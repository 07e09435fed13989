// The C ABI of the tuned SGEMM library: dispatch of a GEMM call to a generated variant, the
// tuning harness (fresh operands, verification against the reference kernel, warm-up and
// median-of-N timing), the per-shape best-configuration cache, and the host-only queries.
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <tuple>
#include <unordered_map>
#include <vector>

#include "../../include/sgemm_tuned.h"
#include "internal.h"
#include "kernelgen.h"
#include "space.h"
#include "strategy.h"
#include "util_kernels.h"

using namespace sgemm;
using namespace sgemm::detail;

namespace {

thread_local std::string t_last_error; // detail of the calling thread's last failure

std::mutex g_mu;                  // guards everything below
hipStream_t g_stream = nullptr;   // stream of sgemm_tuned()
std::map<std::string, std::shared_ptr<LoadedKernel>> g_loaded; // by macro string
constexpr size_t kMaxLoaded = 1024;

struct Tuned {
    sgemm_config cfg;
    float ms;
};
using ShapeKey = std::tuple<int, int, int, int>; // M, N, K, layout
std::map<ShapeKey, Tuned> g_tuned;
bool g_tuned_autoloaded = false;

// What a call of sgemm_tuned_on() needs once it has been seen before: the loaded variant and
// its launch plan, found by one hash lookup on integers.  The key holds everything the choice
// depends on: sizes, storage layout, leading dimensions, how far each pointer is aligned (16,
// 8 or 4 bytes: what decides the load vectors), and whether beta is zero (part of the
// pad-or-guard decision).  Entries are dropped whenever the per-shape table changes.
struct DispatchKey {
    int M, N, K, layout, lda, ldb, ldc, flags;
    bool operator==(const DispatchKey &o) const { return std::memcmp(this, &o, sizeof *this) == 0; }
};
struct DispatchKeyHash {
    size_t operator()(const DispatchKey &k) const {
        uint64_t h = 1469598103934665603ull;
        const int *v = &k.M;
        for (int i = 0; i < 8; ++i) { h ^= (uint64_t)(uint32_t)v[i]; h *= 1099511628211ull; }
        return (size_t)h;
    }
};
struct Dispatch {
    std::shared_ptr<LoadedKernel> kernel; // the build that runs on the operands as they are
    sgemm_config chosen;                  // what the per-shape table selected
    int tiles_m = 0, tiles_n = 0;         // grid of workgroup tiles over C
    int parts = 1, k_chunk = 0;           // split K as it applies to this K
    bool padded = false;                  // sgemm_tuned_on() goes through zero-padded copies
};
std::unordered_map<DispatchKey, Dispatch, DispatchKeyHash> g_dispatch;
constexpr size_t kMaxDispatch = 4096;

void tuned_table_changed_locked() { g_dispatch.clear(); }

int align_class(const void *p) {
    const uintptr_t a = (uintptr_t)p;
    return (a % 16 == 0) ? 2 : (a % 8 == 0) ? 1 : 0;
}

std::string library_dir() {
    Dl_info info;
    if (dladdr((const void *)&library_dir, &info) && info.dli_fname) {
        std::string p = info.dli_fname;
        const size_t slash = p.find_last_of('/');
        return (slash == std::string::npos) ? "." : p.substr(0, slash);
    }
    return ".";
}

int load_cache_file_locked(const char *path) {
    FILE *f = std::fopen(path, "r");
    if (!f) return SGEMM_E_IO;
    char line[512];
    int added = 0;
    while (std::fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        int M, N, K, layout;
        float ms;
        Point p;
        p[13] = 1; // older files have no SK column ...
        p[14] = 2; // ... no NS column ...
        p[15] = 1; // ... and no KSW column
        const int got = std::sscanf(line, "%d %d %d %d %f %d %d %d %d %d %d %d %d %d %d %d %d %d %d %d %d", &M,
                                    &N, &K, &layout, &ms, &p[0], &p[1], &p[2], &p[3], &p[4], &p[5],
                                    &p[6], &p[7], &p[8], &p[9], &p[10], &p[11], &p[12], &p[13], &p[14], &p[15]);
        if (got < 18 || got > 21) continue;
        sgemm_config c = from_point(p);
        if (violates_structure(c) || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 ||
            layout > 3)
            continue;
        g_tuned[ShapeKey{M, N, K, layout}] = Tuned{c, ms};
        ++added;
    }
    std::fclose(f);
    tuned_table_changed_locked();
    return added;
}

void autoload_locked() {
    if (g_tuned_autoloaded) return;
    g_tuned_autoloaded = true;
    if (const char *env = std::getenv("SGEMM_TUNED_CONFIGS")) {
        load_cache_file_locked(env);
        return;
    }
    const std::string p = library_dir() + "/../tuned_configs.txt";
    load_cache_file_locked(p.c_str());
}

struct SplitPlan;
SplitPlan plan_split(const sgemm_config &cfg, int K);

// How a configuration's SK is applied to a problem: `parts` workgroups per tile, each summing
// `k_chunk` consecutive k (a multiple of KWG; the last part takes what is left).
struct SplitPlan {
    int parts;
    int k_chunk;
};

// Built-in fallback for shapes without an entry in the per-shape table: the winners of the tuned
// shapes (and two tiles with edges of 5 and 7 times a power of two) serve as templates, and a
// two-parameter cost model per template chooses among them.
// A workgroup of a template sustains `eff` of a CU's matrix peak while it runs and a launch
// costs `fix_us` on top (launch, first slab, epilogue); the 256 CUs take ceil(workgroups / 256)
// workgroups each, so what decides is how the tile grid quantises the problem.  `eff` and
// `fix_us` were fitted to 27 measured shapes from 300 x 200 x 150 to 7168^3, skinny ones included
// (the model's pick was the fastest template on 21 of them and at most 5 % behind on the rest);
// the 160- and 224-wide tiles were added afterwards, from two shapes each.
// `pairs`: two workgroups of the template fit a CU and hide each other's stalls; a lone one
// reaches 0.93 of `eff`.  `max_sk`: split K is considered for the template.
struct Template {
    int mwg, nwg, kwg, mdimc, ndimc, kwi, mfma, grp, ksw;
    double eff, fix_us;
    bool pairs;
    int max_sk;
};
const Template kTemplates[] = {
    {32, 32, 64, 16, 16, 8, 2, 0, 2, 0.603, 4.0, false, 1},
    {64, 64, 64, 16, 16, 8, 1, 1, 2, 0.821, 4.4, true, 16},
    {64, 64, 128, 32, 32, 32, 2, 1, 1, 0.737, 3.7, false, 1},
    {96, 96, 64, 16, 16, 8, 2, 1, 2, 0.784, 3.9, false, 1},
    {128, 64, 32, 16, 16, 8, 1, 0, 1, 0.829, 4.2, false, 1},
    {128, 128, 64, 16, 32, 8, 1, 1, 1, 0.906, 6.6, false, 16},
    {160, 160, 32, 16, 16, 8, 2, 1, 1, 0.860, 22.4, false, 1}, // (two shapes each: 2560^3 and
    {192, 192, 32, 16, 32, 8, 2, 0, 1, 0.897, 6.4, false, 1},
    {224, 224, 32, 16, 16, 8, 2, 1, 1, 0.895, 14.6, false, 1}, //  5120^3, 3584^3 and 7168^3)
    {256, 128, 32, 16, 32, 8, 1, 1, 1, 0.908, 5.6, false, 1},
    {256, 256, 32, 16, 32, 8, 1, 0, 1, 0.943, 8.8, false, 1},
};
constexpr double kCus = 256.0;
constexpr double kCuFlopPerUs = 614400.0;     // 256 FLOP per clock at 2.4 GHz
constexpr double kReduceFixUs = 3.0;          // the reduction kernel of a split-K call ...
constexpr double kReduceBytesPerUs = 4.0e6;   // ... and the rate at which it moves the planes

sgemm_config config_of(const Template &t, int sk) {
    sgemm_config c{};
    c.mwg = t.mwg; c.nwg = t.nwg; c.kwg = t.kwg; c.mdimc = t.mdimc; c.ndimc = t.ndimc;
    c.vwm = 4; c.vwn = 4; c.sa = 1; c.sb = 1; c.pad = 1; c.kwi = t.kwi; c.mfma = t.mfma;
    c.grp = t.grp; c.sk = sk; c.ns = 2; c.ksw = t.ksw;
    return c;
}

// Predicted microseconds of a call with `cfg`, costed with the parameters of template `t`.
double predicted_us(const sgemm_config &cfg, const Template &t, int M, int N, int K) {
    const SplitPlan plan = plan_split(cfg, K);
    const double tiles = (double)((M + cfg.mwg - 1) / cfg.mwg) * (double)((N + cfg.nwg - 1) / cfg.nwg);
    const double per_cu = std::ceil(tiles * plan.parts / kCus);
    const double k_len = plan.parts > 1 ? plan.k_chunk : (double)((K + cfg.kwg - 1) / cfg.kwg) * cfg.kwg;
    const double eff = t.eff * (t.pairs && per_cu < 2.0 ? 0.93 : 1.0);
    double us = t.fix_us + per_cu * 2.0 * cfg.mwg * cfg.nwg * k_len / (kCuFlopPerUs * eff);
    if (plan.parts > 1) us += kReduceFixUs + (plan.parts + 1.0) * M * N * 4.0 / kReduceBytesPerUs;
    return us;
}

sgemm_config default_config(int M, int N, int K, double *cost_us = nullptr) {
    sgemm_config best = config_of(kTemplates[0], 1);
    double best_us = -1.0;
    for (const Template &t : kTemplates) {
        const long long tiles = (long long)((M + t.mwg - 1) / t.mwg) * ((N + t.nwg - 1) / t.nwg);
        // split K where the tiles alone do not fill the CUs and K is long: parts of at least 8 slabs
        const int slabs = (K + t.kwg - 1) / t.kwg;
        const int sk_max = (tiles <= (long long)kCus && K >= 2048) ? std::min(t.max_sk, slabs / 8) : 1;
        for (int sk = 1; sk <= std::max(1, sk_max); sk *= 2) {
            const sgemm_config c = config_of(t, sk);
            const double us = predicted_us(c, t, M, N, K);
            if (best_us < 0.0 || us < best_us) { best_us = us; best = c; }
        }
    }
    if (cost_us) *cost_us = best_us;
    return best;
}

// The template whose parameters cost a configuration that is not one: the same tile if there
// is one, else the nearest tile area.
const Template &template_like(const sgemm_config &c) {
    const Template *best = &kTemplates[0];
    double best_d = -1.0;
    for (const Template &t : kTemplates) {
        if (t.mwg == c.mwg && t.nwg == c.nwg && t.kwg == c.kwg) return t;
        const double d = std::fabs(std::log2((double)t.mwg * t.nwg) - std::log2((double)c.mwg * c.nwg)) +
                         (t.mwg == c.mwg && t.nwg == c.nwg ? 0.0 : 0.01);
        if (best_d < 0.0 || d < best_d) { best_d = d; best = &t; }
    }
    return *best;
}

int select_config_locked(int M, int N, int K, int layout, sgemm_config *out) {
    autoload_locked();
    auto it = g_tuned.find(ShapeKey{M, N, K, layout});
    if (it != g_tuned.end()) { *out = it->second.cfg; return SGEMM_OK; }
    double default_us = 0.0;
    const sgemm_config fallback = default_config(M, N, K, &default_us);
    // The nearest tuned shape of the same layout, by distance between the logarithms of the
    // sizes, may lend its configuration, if the shapes are alike (every size within about a
    // factor of 1.5, or one size within a factor of 2.3).  It does so when the call has the
    // tuned shape's launch geometry (the same grid of tiles and the same split of K: what was
    // measured there holds here), and otherwise when the cost model, which gives a tuned
    // configuration 3 % credit over the template most like it, does not find a template that
    // quantises this problem better.
    constexpr double kNearEnough = 1.5;
    double best = -1.0;
    const sgemm_config *near_cfg = nullptr;
    ShapeKey near_shape{};
    for (auto &kv : g_tuned) {
        if (std::get<3>(kv.first) != layout) continue;
        const double dm = std::log2((double)std::max(M, 1)) - std::log2((double)std::max(std::get<0>(kv.first), 1));
        const double dn = std::log2((double)std::max(N, 1)) - std::log2((double)std::max(std::get<1>(kv.first), 1));
        const double dk = std::log2((double)std::max(K, 1)) - std::log2((double)std::max(std::get<2>(kv.first), 1));
        const double d = dm * dm + dn * dn + dk * dk;
        if (d <= kNearEnough && (best < 0.0 || d < best)) { best = d; near_cfg = &kv.second.cfg; near_shape = kv.first; }
    }
    if (near_cfg) {
        const sgemm_config &c = *near_cfg;
        const int M0 = std::get<0>(near_shape), N0 = std::get<1>(near_shape), K0 = std::get<2>(near_shape);
        const bool same_geometry = (M + c.mwg - 1) / c.mwg == (M0 + c.mwg - 1) / c.mwg &&
                                   (N + c.nwg - 1) / c.nwg == (N0 + c.nwg - 1) / c.nwg &&
                                   plan_split(c, K).parts == plan_split(c, K0).parts;
        if (same_geometry) { *out = c; return SGEMM_OK; }
        if (c.mfma && 0.97 * predicted_us(c, template_like(c), M, N, K) <= default_us) { *out = c; return SGEMM_OK; }
    }
    *out = fallback;
    return SGEMM_OK;
}

int check_gemm_args(int M, int N, int K, const float *A, int lda, const float *B, int ldb,
                    const float *C, int ldc, int layout, bool need_ab) {
    if (M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize) return SGEMM_E_BADARG;
    if (layout < 0 || layout > 3) return SGEMM_E_BADARG;
    if (M == 0 || N == 0) return SGEMM_OK;
    if (!C || ldc < N) return SGEMM_E_BADARG;
    if (need_ab && K > 0) {
        if (!A || !B) return SGEMM_E_BADARG;
        if (lda < ((layout & 1) ? M : K)) return SGEMM_E_BADARG;
        if (ldb < ((layout & 2) ? K : N)) return SGEMM_E_BADARG;
        // a tile of up to 512 stored rows must lie within the 2 GiB that the kernels' 32-bit
        // byte offsets (and the buffer windows they read through) can span
        if (lda > kMaxLeadingDim || ldb > kMaxLeadingDim) return SGEMM_E_BADARG;
    }
    return SGEMM_OK;
}

bool splits_k(const sgemm_config &cfg, int K);

bool aligned_for(const void *p, int ld, int vw) {
    return ((uintptr_t)p % (uintptr_t)(4 * vw)) == 0 && (ld % vw) == 0;
}

// The variant that will really be launched for this call.
VariantKey resolve_variant(const sgemm_config &cfg, int M, int N, int K, const float *A, int lda,
                           const float *B, int ldb, const float *C, int ldc, int layout, float beta) {
    VariantKey key{cfg, layout, 0};
    key.edge = (M % cfg.mwg || N % cfg.nwg || K % cfg.kwg) ? 1 : 0;
    key.splitk = splits_k(cfg, K) ? 1 : 0;
    // C is read at all only for beta != 0; the build that requests it ahead of the main loop is
    // used where a lane has the registers for it (split-K builds leave C to the reduction)
    key.cpf = (beta != 0.0f && !key.splitk && prefetch_of_c_fits(cfg)) ? 1 : 0;
    if (key.cfg.ns == 0) key.cfg.ns = 2;
    // A vector width is kept only if every access it makes is aligned, and, in a guarded build,
    // if no stored row ends inside a vector (a guarded tile load clamps or zeroes whole vectors).
    // Otherwise it is halved until it fits; LDS-direct loads know only 4 floats or 1.
    const int row_a = (layout & 1) ? M : K, row_b = (layout & 2) ? K : N;
    const bool vwn_loads_b = cfg.sb != 0, vwn_stores_c = cfg.mfma == 0;
    auto a_fits = [&](int v) { return aligned_for(A, lda, v) && (!key.edge || row_a % v == 0); };
    auto b_fits = [&](int v) {
        if (vwn_loads_b && !(aligned_for(B, ldb, v) && (!key.edge || row_b % v == 0))) return false;
        if (!vwn_stores_c) return true;
        // with split K the variant stores into workspace planes of M x N floats, not into C
        return key.splitk ? (N % v == 0 && ((long long)M * N) % v == 0) : aligned_for(C, ldc, v);
    };
    if (key.cfg.sa)
        while (key.cfg.vwm > 1 && !a_fits(key.cfg.vwm)) key.cfg.vwm = key.cfg.sa == 2 ? 1 : key.cfg.vwm / 2;
    while (key.cfg.vwn > 1 && !b_fits(key.cfg.vwn)) key.cfg.vwn = key.cfg.sb == 2 ? 1 : key.cfg.vwn / 2;
    // narrower LDS-direct loads mean more of them, which may not leave room for 3 or 4 buffers
    while (key.cfg.ns > 2 && (key.cfg.ns - 2) * direct_loads_per_slab(key.cfg) > kMaxLoadsInFlight)
        --key.cfg.ns;
    // narrowed loads that no longer fit the counter at all: stage through registers instead
    if (direct_loads_per_slab(key.cfg) > kMaxLoadsInFlight) {
        if (key.cfg.sa == 2) key.cfg.sa = 1;
        if (key.cfg.sb == 2) key.cfg.sb = 1;
        key.cfg.ns = 2;
    }
    return key;
}

// Device workspaces: the split-K planes and the zero-padded copies of the pad-and-run path.
// One set per (device, stream), grown on demand and kept, so calls on different streams never
// share a buffer and calls on one stream are ordered by the stream itself.  hipFree waits for
// the device, so a buffer is never released under a kernel that still uses it.  At most
// kMaxWorkspaces sets are kept; the one unused for longest is released for a new stream.
struct StreamWorkspace {
    float *planes = nullptr;
    size_t plane_floats = 0;
    float *pad = nullptr;
    size_t pad_floats = 0;
    uint64_t last_use = 0;
};
std::map<std::pair<int, hipStream_t>, StreamWorkspace> g_workspaces;
uint64_t g_workspace_clock = 0;
constexpr size_t kMaxWorkspaces = 8;

StreamWorkspace *stream_workspace_locked(hipStream_t s) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    const auto key = std::make_pair(dev, s);
    auto it = g_workspaces.find(key);
    if (it == g_workspaces.end()) {
        if (g_workspaces.size() >= kMaxWorkspaces) {
            auto oldest = g_workspaces.begin();
            for (auto j = g_workspaces.begin(); j != g_workspaces.end(); ++j)
                if (j->second.last_use < oldest->second.last_use) oldest = j;
            if (oldest->second.planes) (void)hipFree(oldest->second.planes);
            if (oldest->second.pad) (void)hipFree(oldest->second.pad);
            g_workspaces.erase(oldest);
        }
        it = g_workspaces.emplace(key, StreamWorkspace{}).first;
    }
    it->second.last_use = ++g_workspace_clock;
    return &it->second;
}

int grow_locked(float **buf, size_t *have, size_t want, size_t at_least, const char *what) {
    if (want <= *have) return SGEMM_OK;
    if (*buf) (void)hipFree(*buf);
    *buf = nullptr;
    *have = 0;
    void *p = nullptr;
    const size_t n = std::max(want, at_least);
    const hipError_t e = hipMalloc(&p, n * sizeof(float));
    if (e != hipSuccess) {
        set_error(std::string("hipMalloc of the ") + what + ": " + hipGetErrorString(e));
        return SGEMM_E_LAUNCH;
    }
    *buf = static_cast<float *>(p);
    *have = n;
    return SGEMM_OK;
}

int workspace_for(hipStream_t s, size_t floats, float **planes) {
    std::lock_guard<std::mutex> lock(g_mu);
    StreamWorkspace *w = stream_workspace_locked(s);
    const int rc = grow_locked(&w->planes, &w->plane_floats, floats, (size_t)(8u << 20), "split-K workspace");
    *planes = w->planes;
    return rc;
}

int pad_workspace_for(hipStream_t s, size_t floats, float **out) {
    std::lock_guard<std::mutex> lock(g_mu);
    StreamWorkspace *w = stream_workspace_locked(s);
    const int rc = grow_locked(&w->pad, &w->pad_floats, floats, 0, "padding workspace");
    *out = w->pad;
    return rc;
}

SplitPlan plan_split(const sgemm_config &cfg, int K) {
    const int slabs = (K + cfg.kwg - 1) / cfg.kwg;
    if (slabs <= 0) return SplitPlan{1, K}; // nothing to sum, nothing to split
    int parts = std::max(1, std::min(cfg.sk, slabs));
    const int chunk_slabs = (slabs + parts - 1) / parts;
    parts = (slabs + chunk_slabs - 1) / chunk_slabs; // no empty parts
    return SplitPlan{parts, parts > 1 ? chunk_slabs * cfg.kwg : K};
}

bool splits_k(const sgemm_config &cfg, int K) { return plan_split(cfg, K).parts > 1; }

// One launch of a loaded variant with its plan worked out: tiles_m x tiles_n tiles of C, `parts`
// workgroups per tile that each sum k_chunk consecutive k into their own plane of `planes`
// (parts * M * N floats of device memory; unused and may be null when parts == 1), followed by
// the reduction kernel when K is split.
int launch_planned(hipStream_t s, const LoadedKernel &k, int tiles_m, int tiles_n, int parts, int k_chunk,
                   float *planes, int M, int N, int K, float alpha, const float *A, int lda, const float *B,
                   int ldb, float beta, float *C, int ldc) {
    const long long wgs = (long long)tiles_m * tiles_n;
    if (wgs > 0x7fffffffll) return SGEMM_E_BADARG;
    void *args[] = {&M, &N, &K, &alpha, &A, &lda, &B, &ldb, &beta, &C, &ldc, &tiles_m, &tiles_n, &k_chunk, &planes};
    const hipError_t e = hipModuleLaunchKernel(k.fn, (unsigned)wgs, (unsigned)parts, 1, (unsigned)k.threads, 1, 1,
                                               0, s, args, nullptr);
    if (e != hipSuccess) {
        set_error(std::string("hipModuleLaunchKernel: ") + hipGetErrorString(e));
        return SGEMM_E_LAUNCH;
    }
    if (parts > 1) {
        const hipError_t r = sgemm_util::launch_splitk_reduce(s, M, N, parts, planes, (size_t)M * (size_t)N, alpha,
                                                              beta, C, ldc);
        if (r != hipSuccess) {
            set_error(std::string("split-K reduction: ") + hipGetErrorString(r));
            return SGEMM_E_LAUNCH;
        }
    }
    return SGEMM_OK;
}

int launch_loaded(hipStream_t s, const LoadedKernel &k, const sgemm_config &cfg, int M, int N, int K,
                  float alpha, const float *A, int lda, const float *B, int ldb, float beta, float *C,
                  int ldc) {
    const SplitPlan plan = plan_split(cfg, K);
    float *planes = nullptr;
    if (plan.parts > 1) {
        const int rc = workspace_for(s, (size_t)plan.parts * (size_t)M * (size_t)N, &planes);
        if (rc != SGEMM_OK) return rc;
    }
    return launch_planned(s, k, (M + cfg.mwg - 1) / cfg.mwg, (N + cfg.nwg - 1) / cfg.nwg, plan.parts, plan.k_chunk,
                          planes, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
}

int get_loaded(const VariantKey &key, std::shared_ptr<LoadedKernel> *out) {
    const std::string name = key.macros();
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_loaded.find(name);
        if (it != g_loaded.end()) { *out = it->second; return SGEMM_OK; }
    }
    std::string log;
    std::shared_ptr<LoadedKernel> k;
    const int rc = load_kernel(key, &k, &log);
    if (rc != SGEMM_OK) {
        set_error(log);
        return rc;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_loaded.size() >= kMaxLoaded) {
        (void)hipDeviceSynchronize(); // no variant may still be running when its module goes away
        g_loaded.clear();
    }
    g_loaded[name] = k;
    *out = std::move(k);
    return SGEMM_OK;
}

int run_config(hipStream_t s, const sgemm_config &cfg, int M, int N, int K, float alpha,
               const float *A, int lda, const float *B, int ldb, float beta, float *C, int ldc,
               int layout) {
    const bool need_ab = (alpha != 0.0f);
    int rc = check_gemm_args(M, N, K, A, lda, B, ldb, C, ldc, layout, need_ab);
    if (rc != SGEMM_OK) return rc;
    if (violates_structure(cfg)) return SGEMM_E_INVALID;
    if (M == 0 || N == 0) return SGEMM_OK;
    if (K == 0 || alpha == 0.0f) {
        if (beta == 1.0f) return SGEMM_OK;
        return sgemm_util::launch_scale(s, M, N, beta, C, ldc) == hipSuccess ? SGEMM_OK : SGEMM_E_LAUNCH;
    }
    const VariantKey key = resolve_variant(cfg, M, N, K, A, lda, B, ldb, C, ldc, layout, beta);
    std::shared_ptr<LoadedKernel> k;
    rc = get_loaded(key, &k);
    if (rc != SGEMM_OK) return rc;
    return launch_loaded(s, *k, key.cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
}

void fill_result(const Space &space, const SearchResult &r, double flops, tune_result *out) {
    if (!out) return;
    *out = tune_result{};
    out->best_index = r.best_index;
    out->evaluations = r.evaluations;
    out->failed = r.failed;
    out->space_size = (int)space.configs.size();
    out->evals_to_best = r.evals_to_best;
    if (r.best_index >= 0) {
        out->best = from_point(space.configs[r.best_index]);
        out->best_ms = (float)r.best_cost;
        out->best_gflops = (float)(flops / (r.best_cost * 1e-3) * 1e-9);
    }
}

// ---- on-line tuning ------------------------------------------------------------------------
// The paper also proposes tuning at run time, in the first calls of an application ("CLTune:
// an auto-tuner for OpenCL kernels").  One search per problem shape runs in a thread of its
// own; its cost function hands the next configuration to the GEMM call that is waiting for
// one and blocks until that call reports the time it measured, so the four strategies are
// used exactly as they are.
struct OnlineSearch {
    std::mutex mu;
    std::condition_variable cv;
    std::thread worker;
    int wanted = -1;        // configuration the search wants timed next (-1: none yet)
    bool taken = false;     // a GEMM call has picked `wanted` up and is timing it
    double reported = 0.0;  // its time, once has_report is set
    bool has_report = false;
    bool finished = false;  // the search has ended; best_index holds its result
    bool abandoned = false; // the library is shutting the search down
    int best_index = -1;
    double best_ms = 0.0;
    int evaluations = 0;

    ~OnlineSearch() {
        {
            std::lock_guard<std::mutex> lock(mu);
            abandoned = true;
        }
        cv.notify_all();
        if (worker.joinable()) worker.join();
    }
};
std::mutex g_online_mu;
// (shared: a call keeps its search alive while it waits on it, whoever removes the entry)
std::map<std::tuple<int, int, int, int, int>, std::shared_ptr<OnlineSearch>> g_online; // + space

} // namespace

namespace sgemm {
namespace detail {

void set_error(const std::string &what) {
    t_last_error = what;
    if (std::getenv("SGEMM_TUNED_VERBOSE")) std::fprintf(stderr, "sgemm_tuned: %s\n", what.c_str());
}

hipStream_t library_stream() {
    std::lock_guard<std::mutex> lock(g_mu);
    return g_stream;
}

double median(std::vector<double> v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n % 2 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

StrategyParams params_from(const tune_opts *o) {
    StrategyParams p;
    if (!o) return p;
    if (o->sa_T > 0) p.sa_T = o->sa_T;
    p.sa_raw_ms = o->sa_raw_ms != 0;
    if (o->pso_S > 0) p.pso_S = o->pso_S;
    if (o->pso_alpha != 0 || o->pso_beta != 0 || o->pso_gamma != 0) {
        p.pso_alpha = o->pso_alpha; p.pso_beta = o->pso_beta; p.pso_gamma = o->pso_gamma;
    }
    if (o->random_fraction > 0) p.random_fraction = o->random_fraction;
    if (o->warm_start < 0) p.start_index = -o->warm_start - 1;
    return p;
}

TimingRules timing_rules_from(const tune_opts *o) {
    TimingRules r;
    if (o && o->warmup > 0) r.warmup = o->warmup;
    if (o && o->reps > 0) r.reps = o->reps;
    if (o && o->cut_factor != 0.0f) r.cut = o->cut_factor;
    if (o && o->warmup_ms != 0.0f) r.warmup_ms = o->warmup_ms;
    return r;
}

double time_configuration(hipStream_t s, const std::function<void()> &launch, float first,
                          const TimingRules &rules, double best_ms, Event &ev0, Event &ev1,
                          int *samples, bool *was_cut) {
    *was_cut = false;
    // `first` is the duration of the verified launch: cold clocks, up to ~1.25x slow
    if (rules.cut > 0.0 && best_ms > 0.0 && first > 1.3 * rules.cut * best_ms) {
        *samples = 1; // hopeless even allowing for the cold start: not worth warming up
        *was_cut = true;
        return first;
    }
    int warm = rules.warmup - 1;
    if (rules.warmup_ms > 0.0 && first > 0.0f)
        warm = std::max(warm, std::min(4096, (int)std::ceil(rules.warmup_ms / first)));
    for (int w = 0; w < warm; ++w) launch();
    // short kernels: several launches per sample so that a sample lasts >= 0.2 ms
    int batch = 1;
    if (first > 0.0f && first < 0.2f) batch = std::min(64, (int)std::ceil(0.2f / first));
    std::vector<double> t;
    for (int r = 0; r < rules.reps; ++r) {
        (void)hipEventRecord(ev0.e, s);
        for (int b = 0; b < batch; ++b) launch();
        (void)hipEventRecord(ev1.e, s);
        if (hipEventSynchronize(ev1.e) != hipSuccess) return -1.0;
        float e = 0.0f;
        (void)hipEventElapsedTime(&e, ev0.e, ev1.e);
        t.push_back((double)e / batch);
        if (r == 0 && rules.cut > 0.0 && best_ms > 0.0 && t[0] > rules.cut * best_ms) {
            *was_cut = true;
            break;
        }
    }
    if (t.empty()) return -1.0;
    *samples = (int)t.size();
    return median(t);
}

Measured run_verify_time(hipStream_t s, const std::function<void()> &fresh_arguments,
                         const std::function<bool()> &launch, const std::function<int()> &outputs_differ,
                         const TimingRules &rules, double best_ms, Event &ev0, Event &ev1) {
    Measured m;
    if (fresh_arguments) fresh_arguments();
    (void)hipEventRecord(ev0.e, s);
    if (!launch()) { m.status = "launch"; return m; }
    (void)hipEventRecord(ev1.e, s);
    const int differ = outputs_differ ? outputs_differ() : (hipStreamSynchronize(s) == hipSuccess ? 0 : -1);
    if (differ < 0) { m.status = "fault"; m.device_failed = true; return m; }
    if (differ > 0) { m.status = "verify"; return m; }
    float first = 0.0f;
    (void)hipEventElapsedTime(&first, ev0.e, ev1.e);
    bool was_cut = false;
    m.ms = time_configuration(s, [&] { (void)launch(); }, first, rules, best_ms, ev0, ev1, &m.samples, &was_cut);
    if (m.ms < 0.0) { m.status = "fault"; m.device_failed = true; return m; }
    if (was_cut) m.status = "ok-cut";
    return m;
}

} // namespace detail
} // namespace sgemm

extern "C" {

const char *sgemm_last_error(void) { return t_last_error.c_str(); }

const char *sgemm_status_string(int status) {
    switch (status) {
    case SGEMM_OK: return "ok";
    case SGEMM_E_BADARG: return "bad argument";
    case SGEMM_E_NOCONFIG: return "no configuration";
    case SGEMM_E_COMPILE: return "kernel compilation failed";
    case SGEMM_E_LAUNCH: return "HIP call failed";
    case SGEMM_E_VERIFY: return "verification against the reference kernel failed";
    case SGEMM_E_INVALID: return "configuration violates a constraint";
    case SGEMM_E_IO: return "cache file i/o failed";
    case SGEMM_E_NODEVICE: return "no HIP device";
    case SGEMM_E_RESOURCE: return "variant spills registers or exceeds LDS, or scratch memory too small";
    case SGEMM_E_NOTREADY: return "call not prepared (no allocation allowed)";
    default: return status > 0 ? "count" : "unknown status";
    }
}

int sgemm_set_stream(void *hip_stream) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_stream = static_cast<hipStream_t>(hip_stream);
    return SGEMM_OK;
}

int sgemm_run_config(void *hip_stream, const sgemm_config *cfg, int M, int N, int K, float alpha,
                     const float *A, int lda, const float *B, int ldb, float beta, float *C, int ldc,
                     int layout) {
    if (!cfg) return SGEMM_E_BADARG;
    return run_config(static_cast<hipStream_t>(hip_stream), *cfg, M, N, K, alpha, A, lda, B, ldb,
                      beta, C, ldc, layout);
}

int sgemm_run_config_padded(void *hip_stream, const sgemm_config *cfg, int M, int N, int K,
                            float alpha, const float *A, int lda, const float *B, int ldb, float beta,
                            float *C, int ldc, int layout) {
    if (!cfg) return SGEMM_E_BADARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int rc = check_gemm_args(M, N, K, A, lda, B, ldb, C, ldc, layout, alpha != 0.0f);
    if (rc != SGEMM_OK) return rc;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    const int Mp = (M + cfg->mwg - 1) / cfg->mwg * cfg->mwg;
    const int Np = (N + cfg->nwg - 1) / cfg->nwg * cfg->nwg;
    const int Kp = (K + cfg->kwg - 1) / cfg->kwg * cfg->kwg;
    // nothing to pad, or nothing to multiply: the ordinary path
    if ((Mp == M && Np == N && Kp == K) || M == 0 || N == 0 || K == 0 || alpha == 0.0f)
        return run_config(s, *cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout);
    const int a_rows = (layout & 1) ? K : M, a_cols = (layout & 1) ? M : K;
    const int b_rows = (layout & 2) ? N : K, b_cols = (layout & 2) ? K : N;
    const int ap_rows = (layout & 1) ? Kp : Mp, ap_cols = (layout & 1) ? Mp : Kp;
    const int bp_rows = (layout & 2) ? Np : Kp, bp_cols = (layout & 2) ? Kp : Np;
    const size_t na = (size_t)ap_rows * ap_cols, nb = (size_t)bp_rows * bp_cols, nc = (size_t)Mp * Np;
    float *ws = nullptr;
    rc = pad_workspace_for(s, na + nb + nc, &ws);
    if (rc != SGEMM_OK) return rc;
    float *Ap = ws, *Bp = ws + na, *Cp = ws + na + nb;
    hipError_t e = sgemm_util::launch_pad_copy(s, Ap, ap_cols, ap_rows, ap_cols, A, lda, a_rows, a_cols);
    if (e == hipSuccess) e = sgemm_util::launch_pad_copy(s, Bp, bp_cols, bp_rows, bp_cols, B, ldb, b_rows, b_cols);
    // C' needs the old C only when beta != 0 (its padding is never copied back)
    if (e == hipSuccess && beta != 0.0f) e = sgemm_util::launch_pad_copy(s, Cp, Np, Mp, Np, C, ldc, M, N);
    if (e != hipSuccess) {
        set_error(std::string("padding copy: ") + hipGetErrorString(e));
        return SGEMM_E_LAUNCH;
    }
    rc = run_config(s, *cfg, Mp, Np, Kp, alpha, Ap, ap_cols, Bp, bp_cols, beta, Cp, Np, layout);
    if (rc != SGEMM_OK) return rc;
    e = sgemm_util::launch_copy2d(s, C, ldc, Cp, Np, M, N);
    if (e != hipSuccess) {
        set_error(std::string("copy of the result out of the padded buffer: ") + hipGetErrorString(e));
        return SGEMM_E_LAUNCH;
    }
    return SGEMM_OK;
}

// Guarded build on the operands as they are, or zero-padded copies and the unguarded build?
// The guarded build costs little unless a stored row is not a multiple of the load vector: then
// its loads are narrowed, and with the 4096^3 winner it runs at about 0.93 of the unguarded rate
// with 2-float loads (rows even: measured 134.5 against 144.5 TFLOP/s at 4090^3) and 0.86 with
// single floats (rows odd: 122.7 at 4091^3).  The padded path pays four extra launches and copies
// that run at about half the HBM rate (measured 4.2 TB/s).  Padding is chosen when this model
// says it wins by more than 3 %: odd row lengths from about 3800^3 upwards for beta = 0 and
// 4900^3 for beta != 0.
bool prefers_padding(const sgemm_config &cfg, int M, int N, int K, const float *A, int lda, const float *B,
                     int ldb, const float *C, int ldc, int layout, float alpha, float beta) {
    if (M == 0 || N == 0 || K == 0 || alpha == 0.0f) return false;
    const VariantKey key = resolve_variant(cfg, M, N, K, A, lda, B, ldb, C, ldc, layout, beta);
    if (!key.edge) return false;
    auto rate_with = [](int wanted, int got) { return wanted < 4 || got >= 4 ? 1.0 : got == 2 ? 0.93 : 0.86; };
    double rate = 1.0;
    if (cfg.sa) rate = std::min(rate, rate_with(cfg.vwm, key.cfg.vwm));
    if (cfg.sb) rate = std::min(rate, rate_with(cfg.vwn, key.cfg.vwn));
    if (rate == 1.0) return false;
    const double Mp = (M + cfg.mwg - 1) / cfg.mwg * (double)cfg.mwg, Np = (N + cfg.nwg - 1) / cfg.nwg * (double)cfg.nwg,
                 Kp = (K + cfg.kwg - 1) / cfg.kwg * (double)cfg.kwg;
    const double t_guarded = 2.0 * M * N * (double)K / (rate * 145e12);
    const double t_unguarded = 2.0 * Mp * Np * Kp / 145e12;
    const double copied = 4.0 * (2.0 * (Mp * Kp + Kp * Np) + (beta != 0.0f ? 2.0 * Mp * Np : 0.0) + 2.0 * M * (double)N);
    const double t_copies = copied / 4.2e12 + 12e-6;
    return t_guarded > 1.03 * (t_unguarded + t_copies);
}

// The slow half of a dispatch: choose the configuration, decide between the guarded build and
// zero-padded copies, resolve and load the variant, work out the launch plan.
static int build_dispatch(int M, int N, int K, float alpha, const float *A, int lda, const float *B, int ldb,
                          float beta, const float *C, int ldc, int layout, Dispatch *d) {
    {
        std::lock_guard<std::mutex> lock(g_mu);
        select_config_locked(M, N, K, layout, &d->chosen);
    }
    d->padded = prefers_padding(d->chosen, M, N, K, A, lda, B, ldb, C, ldc, layout, alpha, beta);
    const VariantKey key = resolve_variant(d->chosen, M, N, K, A, lda, B, ldb, C, ldc, layout, beta);
    const int rc = get_loaded(key, &d->kernel);
    if (rc != SGEMM_OK) return rc;
    const SplitPlan plan = plan_split(key.cfg, K);
    d->tiles_m = (M + key.cfg.mwg - 1) / key.cfg.mwg;
    d->tiles_n = (N + key.cfg.nwg - 1) / key.cfg.nwg;
    d->parts = plan.parts;
    d->k_chunk = plan.k_chunk;
    return SGEMM_OK;
}

// Shared by sgemm_tuned_on() and sgemm_tuned_noalloc().  `may_allocate` = false: a call that
// has not been seen before (its variant would have to be loaded) is an error, zero-padded copies
// are never used, and the split-K planes lie in the library's static device array.
static int dispatch_call(hipStream_t s, int M, int N, int K, float alpha, const float *A, int lda, const float *B,
                         int ldb, float beta, float *C, int ldc, int layout, bool may_allocate) {
    const int rc0 = check_gemm_args(M, N, K, A, lda, B, ldb, C, ldc, layout, alpha != 0.0f);
    if (rc0 != SGEMM_OK) return rc0;
    if (M == 0 || N == 0) return SGEMM_OK;
    if (K == 0 || alpha == 0.0f) {
        if (beta == 1.0f) return SGEMM_OK;
        return sgemm_util::launch_scale(s, M, N, beta, C, ldc) == hipSuccess ? SGEMM_OK : SGEMM_E_LAUNCH;
    }
    const DispatchKey key{M, N, K, layout, lda, ldb, ldc,
                          align_class(A) | (align_class(B) << 2) | (align_class(C) << 4) | (beta == 0.0f ? 64 : 0)};
    Dispatch d;
    bool hit;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_dispatch.find(key);
        hit = it != g_dispatch.end();
        if (hit) d = it->second;
    }
    if (!hit) {
        if (!may_allocate) {
            set_error("this call has not been prepared: make the same call (sizes, leading dimensions, storage "
                      "layout, pointer alignment, beta zero or not) once through sgemm_tuned_on() first");
            return SGEMM_E_NOTREADY;
        }
        const int rc = build_dispatch(M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout, &d);
        if (rc != SGEMM_OK) return rc;
        std::lock_guard<std::mutex> lock(g_mu);
        if (g_dispatch.size() >= kMaxDispatch) g_dispatch.clear();
        g_dispatch[key] = d;
    }
    float *planes = nullptr;
    if (may_allocate) {
        if (d.padded)
            return sgemm_run_config_padded(s, &d.chosen, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout);
        if (d.parts > 1) {
            const int rc = workspace_for(s, (size_t)d.parts * (size_t)M * (size_t)N, &planes);
            if (rc != SGEMM_OK) return rc;
        }
    } else if (d.parts > 1) {
        const size_t need = (size_t)d.parts * (size_t)M * (size_t)N;
        if (need > sgemm_util::kScratchFloats) {
            char msg[256];
            std::snprintf(msg, sizeof msg,
                          "split K of this call needs %d planes of %d x %d floats = %zu bytes, more than the %zu "
                          "bytes of static device scratch memory: use sgemm_tuned_on()",
                          d.parts, M, N, need * sizeof(float), sgemm_util::kScratchFloats * sizeof(float));
            set_error(msg);
            return SGEMM_E_RESOURCE;
        }
        const hipError_t e = sgemm_util::scratch_of_current_device(&planes);
        if (e != hipSuccess) {
            set_error(std::string("address of the static scratch array: ") + hipGetErrorString(e));
            return SGEMM_E_LAUNCH;
        }
    }
    return launch_planned(s, *d.kernel, d.tiles_m, d.tiles_n, d.parts, d.k_chunk, planes, M, N, K, alpha, A, lda, B,
                          ldb, beta, C, ldc);
}

int sgemm_tuned_on(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                   const float *B, int ldb, float beta, float *C, int ldc, int layout) {
    return dispatch_call(static_cast<hipStream_t>(hip_stream), M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout,
                         true);
}

int sgemm_tuned_noalloc(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                        const float *B, int ldb, float beta, float *C, int ldc, int layout) {
    return dispatch_call(static_cast<hipStream_t>(hip_stream), M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout,
                         false);
}

static_assert(sgemm_util::kScratchFloats * sizeof(float) == SGEMM_NOALLOC_SCRATCH_BYTES,
              "the header states the size of the static scratch array");

int sgemm_config_prefers_padding(const sgemm_config *cfg, int M, int N, int K, int lda, int ldb, int ldc,
                                 int layout, float beta) {
    if (!cfg || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    const float *aligned = reinterpret_cast<const float *>(uintptr_t{256});
    return prefers_padding(*cfg, M, N, K, aligned, lda, aligned, ldb, aligned, ldc, layout, 1.0f, beta) ? 1 : 0;
}

int sgemm_tuned_online(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                       const float *B, int ldb, float beta, float *C, int ldc, int layout,
                       int space_id, int strategy, int budget) {
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int rc0 = check_gemm_args(M, N, K, A, lda, B, ldb, C, ldc, layout, alpha != 0.0f);
    if (rc0 != SGEMM_OK) return rc0;
    const Space *space = get_space(space_id);
    if (!space || strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    if (space->configs.empty()) return SGEMM_E_NOCONFIG;
    // nothing to time, or already tuned: the ordinary asynchronous call
    bool tuned;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        autoload_locked();
        tuned = g_tuned.count(ShapeKey{M, N, K, layout}) != 0;
    }
    if (tuned || M == 0 || N == 0 || K == 0 || alpha == 0.0f || budget <= 0)
        return sgemm_tuned_on(hip_stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout);

    std::shared_ptr<OnlineSearch> os;
    {
        std::lock_guard<std::mutex> lock(g_online_mu);
        auto &slot = g_online[std::make_tuple(M, N, K, layout, space_id)];
        if (!slot) {
            slot = std::make_shared<OnlineSearch>();
            OnlineSearch *self = slot.get();
            const uint64_t seed = ((uint64_t)M * 1000003ull + (uint64_t)N) * 1000003ull + (uint64_t)K + (uint64_t)layout;
            self->worker = std::thread([self, space, strategy, budget, seed] {
                const SearchResult r = run_search(*space, strategy, budget, seed, StrategyParams{}, [self](int idx) {
                    std::unique_lock<std::mutex> lock(self->mu);
                    self->wanted = idx;
                    self->taken = false;
                    self->has_report = false;
                    self->cv.notify_all();
                    self->cv.wait(lock, [self] { return self->has_report || self->abandoned; });
                    self->wanted = -1;
                    return self->abandoned ? -1.0 : self->reported;
                });
                std::lock_guard<std::mutex> lock(self->mu);
                self->best_index = r.best_index;
                self->best_ms = r.best_cost;
                self->evaluations = r.evaluations;
                self->finished = true;
                self->cv.notify_all();
            });
        }
        os = slot;
    }

    // One GEMM per call, done by the next candidate that compiles and launches; a candidate
    // that does not is reported as failed and the search is asked for another one.
    Event ev0, ev1;
    for (;;) {
        int idx;
        {
            std::unique_lock<std::mutex> lock(os->mu);
            // one call per candidate: concurrent calls of the same shape wait for the next one
            os->cv.wait(lock, [&os] { return os->finished || (os->wanted >= 0 && !os->has_report && !os->taken); });
            if (os->finished) break;
            idx = os->wanted;
            os->taken = true;
        }
        const sgemm_config cfg = from_point(space->configs[idx]);
        double ms = -1.0;
        int launched = SGEMM_E_LAUNCH;
        do {
            const VariantKey key = resolve_variant(cfg, M, N, K, A, lda, B, ldb, C, ldc, layout, beta);
            std::shared_ptr<LoadedKernel> k;
            if (get_loaded(key, &k) != SGEMM_OK) break;
            if (k->info.scratch_bytes > 0 || k->info.lds_bytes > kLdsLimitBytes) break;
            (void)hipEventRecord(ev0.e, s);
            launched = launch_loaded(s, *k, key.cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc);
            if (launched != SGEMM_OK) break;
            (void)hipEventRecord(ev1.e, s);
            if (hipEventSynchronize(ev1.e) != hipSuccess) { launched = SGEMM_E_LAUNCH; break; }
            float e = 0.0f;
            (void)hipEventElapsedTime(&e, ev0.e, ev1.e);
            ms = e;
        } while (false);
        {
            std::lock_guard<std::mutex> lock(os->mu);
            os->reported = ms;
            os->has_report = true;
        }
        os->cv.notify_all();
        if (launched == SGEMM_OK) return SGEMM_OK; // this call's GEMM is done
    }
    // the search is over: keep its winner, drop the search, and serve this call normally
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (os->best_index >= 0) {
            g_tuned[ShapeKey{M, N, K, layout}] = Tuned{from_point(space->configs[os->best_index]), (float)os->best_ms};
        } else {
            // nothing in the space worked here: settle on what the dispatch would pick anyway,
            // so that the next call does not start the search over
            sgemm_config fallback;
            select_config_locked(M, N, K, layout, &fallback);
            g_tuned[ShapeKey{M, N, K, layout}] = Tuned{fallback, 0.0f};
        }
        tuned_table_changed_locked();
    }
    {
        std::lock_guard<std::mutex> lock(g_online_mu);
        auto it = g_online.find(std::make_tuple(M, N, K, layout, space_id));
        if (it != g_online.end() && it->second == os) g_online.erase(it);
    }
    return sgemm_tuned_on(hip_stream, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout);
}

int sgemm_tuned(int M, int N, int K, float alpha, const float *A, int lda, const float *B, int ldb,
                float beta, float *C, int ldc, int layout) {
    hipStream_t s;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        s = g_stream;
    }
    return sgemm_tuned_on(s, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, layout);
}

int sgemm_reference(void *hip_stream, int M, int N, int K, float alpha, const float *A, int lda,
                    const float *B, int ldb, float beta, float *C, int ldc, int layout) {
    const int rc = check_gemm_args(M, N, K, A, lda, B, ldb, C, ldc, layout, alpha != 0.0f);
    if (rc != SGEMM_OK) return rc;
    return sgemm_util::launch_reference(static_cast<hipStream_t>(hip_stream), M, N, K, alpha, A, lda, B,
                                        ldb, beta, C, ldc, layout) == hipSuccess
               ? SGEMM_OK
               : SGEMM_E_LAUNCH;
}

/* ---- search space ------------------------------------------------------------------- */

int sgemm_space_define_custom(const char *spec) {
    const int n = define_custom_space(spec);
    return n < 0 ? SGEMM_E_BADARG : n;
}

int sgemm_space_size(int space) {
    const Space *s = get_space(space);
    return s ? (int)s->configs.size() : SGEMM_E_BADARG;
}

long long sgemm_space_raw_size(int space) {
    const Space *s = get_space(space);
    return s ? s->raw : SGEMM_E_BADARG;
}

int sgemm_space_get(int space, int index, sgemm_config *out) {
    const Space *s = get_space(space);
    if (!s || !out || index < 0 || index >= (int)s->configs.size()) return SGEMM_E_BADARG;
    *out = from_point(s->configs[index]);
    return SGEMM_OK;
}

int sgemm_space_find(int space, const sgemm_config *cfg) {
    const Space *s = get_space(space);
    if (!s || !cfg) return SGEMM_E_BADARG;
    const int i = s->find(to_point(*cfg));
    return i >= 0 ? i : SGEMM_E_INVALID;
}

int sgemm_space_dims(int space) { return get_space(space) ? kDims : SGEMM_E_BADARG; }

int sgemm_space_values(int space, int dim, int *values, int cap) {
    const Space *s = get_space(space);
    if (!s || dim < 0 || dim >= kDims) return SGEMM_E_BADARG;
    const auto &v = s->values[dim];
    for (int i = 0; i < (int)v.size() && i < cap && values; ++i) values[i] = v[i];
    return (int)v.size();
}

int sgemm_config_check(const sgemm_config *cfg) {
    if (!cfg) return SGEMM_E_BADARG;
    return violates(*cfg) ? SGEMM_E_INVALID : SGEMM_OK;
}

int sgemm_config_lds_bytes(const sgemm_config *cfg) {
    if (!cfg) return SGEMM_E_BADARG;
    return lds_bytes(*cfg);
}

long long sgemm_config_workspace_bytes(const sgemm_config *cfg, int M, int N, int K, int *parts,
                                       int *k_chunk) {
    if (!cfg || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize) return SGEMM_E_BADARG;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    const SplitPlan plan = plan_split(*cfg, K);
    if (parts) *parts = plan.parts;
    if (k_chunk) *k_chunk = plan.k_chunk;
    return plan.parts > 1 ? (long long)plan.parts * M * N * 4 : 0;
}

int sgemm_config_default(int M, int N, int K, int layout, sgemm_config *out) {
    if (!out || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    *out = default_config(M, N, K);
    return SGEMM_OK;
}

/* ---- kernel generator ---------------------------------------------------------------- */

int sgemm_kernel_cache_dir(const char *path) {
    if (!path || !*path) return SGEMM_E_BADARG;
    set_cache_dir(path);
    return SGEMM_OK;
}

// The build that the query functions' `build` flags name.
static VariantKey named_build(const sgemm_config &cfg, int layout, int build) {
    VariantKey key{cfg, layout, (build & SGEMM_BUILD_GUARDED) ? 1 : 0, cfg.sk > 1 ? 1 : 0};
    key.cpf = (build & SGEMM_BUILD_READS_C_AHEAD) && !key.splitk && cfg.mfma ? 1 : 0;
    return key;
}

int sgemm_kernel_compile(const sgemm_config *cfg, int layout, int edge, sgemm_kernel_info *info) {
    if (!cfg || layout < 0 || layout > 3) return SGEMM_E_BADARG;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    CodeObject co;
    std::string log;
    const int rc = get_code_object(named_build(*cfg, layout, edge), &co, &log);
    if (rc != SGEMM_OK) set_error(log);
    if (info) *info = co.info;
    return rc;
}

int sgemm_kernel_resolve(const sgemm_config *cfg, int M, int N, int K, int lda, int ldb, int ldc,
                         int layout, float beta, sgemm_config *variant, int *build) {
    if (!cfg || !variant || !build || M <= 0 || N <= 0 || K <= 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize ||
        layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    const float *aligned = reinterpret_cast<const float *>(uintptr_t{256}); // stands for any aligned pointer
    const VariantKey key = resolve_variant(*cfg, M, N, K, aligned, lda, aligned, ldb, aligned, ldc, layout, beta);
    *variant = key.cfg;
    variant->sk = key.splitk ? std::max(2, cfg->sk) : 1;
    *build = (key.edge ? SGEMM_BUILD_GUARDED : 0) | (key.cpf ? SGEMM_BUILD_READS_C_AHEAD : 0);
    return SGEMM_OK;
}

int sgemm_kernel_cache_path(const sgemm_config *cfg, int layout, int edge, char *buf, int cap) {
    if (!cfg || !buf || cap <= 0 || layout < 0 || layout > 3) return SGEMM_E_BADARG;
    if (violates_structure(*cfg)) return SGEMM_E_INVALID;
    const std::string p = code_object_path(named_build(*cfg, layout, edge));
    if ((int)p.size() + 1 > cap) return SGEMM_E_BADARG;
    std::memcpy(buf, p.c_str(), p.size() + 1);
    return SGEMM_OK;
}

int sgemm_kernel_macros(const sgemm_config *cfg, int layout, int edge, char *buf, int cap) {
    if (!cfg || !buf || cap <= 0) return SGEMM_E_BADARG;
    const std::string m = named_build(*cfg, layout, edge).macros();
    if ((int)m.size() + 1 > cap) return SGEMM_E_BADARG;
    std::memcpy(buf, m.c_str(), m.size() + 1);
    return SGEMM_OK;
}

/* ---- per-shape cache ------------------------------------------------------------------ */

int sgemm_config_get(int M, int N, int K, int layout, sgemm_config *out) {
    if (!out) return SGEMM_E_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    autoload_locked();
    auto it = g_tuned.find(ShapeKey{M, N, K, layout});
    if (it == g_tuned.end()) return SGEMM_E_NOCONFIG;
    *out = it->second.cfg;
    return SGEMM_OK;
}

int sgemm_config_set(int M, int N, int K, int layout, const sgemm_config *cfg, float ms) {
    if (!cfg || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    if (violates(*cfg)) return SGEMM_E_INVALID;
    std::lock_guard<std::mutex> lock(g_mu);
    autoload_locked();
    g_tuned[ShapeKey{M, N, K, layout}] = Tuned{*cfg, ms};
    tuned_table_changed_locked();
    return SGEMM_OK;
}

int sgemm_config_select(int M, int N, int K, int layout, sgemm_config *out) {
    if (!out || M < 0 || N < 0 || K < 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    return select_config_locked(M, N, K, layout, out);
}

int sgemm_cache_load(const char *path) {
    if (!path) return SGEMM_E_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    autoload_locked();
    const int rc = load_cache_file_locked(path);
    return rc < 0 ? rc : SGEMM_OK;
}

int sgemm_cache_save(const char *path) {
    if (!path) return SGEMM_E_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    autoload_locked();
    FILE *f = std::fopen(path, "w");
    if (!f) return SGEMM_E_IO;
    std::fprintf(f, "# M N K layout ms MWG NWG KWG MDIMC NDIMC VWM VWN SA SB PAD KWI MFMA GRP SK NS KSW\n");
    for (auto &kv : g_tuned) {
        const Point p = to_point(kv.second.cfg);
        std::fprintf(f, "%d %d %d %d %.6g", std::get<0>(kv.first), std::get<1>(kv.first),
                     std::get<2>(kv.first), std::get<3>(kv.first), kv.second.ms);
        for (int v : p) std::fprintf(f, " %d", v);
        std::fprintf(f, "\n");
    }
    return std::fclose(f) == 0 ? SGEMM_OK : SGEMM_E_IO;
}

int sgemm_cache_clear(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_tuned_autoloaded = true; // an explicit clear also drops the auto-loaded entries
    g_tuned.clear();
    tuned_table_changed_locked();
    return SGEMM_OK;
}

int sgemm_cache_count(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    autoload_locked();
    return (int)g_tuned.size();
}

/* ---- device facts ---------------------------------------------------------------------- */

int sgemm_device_peak(float *gflops, int *compute_units, int *clock_mhz) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SGEMM_E_NODEVICE;
    int cus = 0, khz = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess)
        return SGEMM_E_NODEVICE;
    if (compute_units) *compute_units = cus;
    if (clock_mhz) *clock_mhz = khz / 1000;
    // 4 SIMDs x (one 32x32x2 fp32 MFMA = 4096 FLOP per 64 cycles) = 256 FLOP per clock per CU
    if (gflops) *gflops = (float)((double)cus * 256.0 * (double)khz * 1e-6);
    return SGEMM_OK;
}

/* ---- tuning ------------------------------------------------------------------------------ */

int tune_replay(int space_id, const float *ms_table, int table_len, int strategy, int budget,
                unsigned long long seed, const tune_opts *opts, int *visited, int visited_cap,
                tune_result *out) {
    const Space *space = get_space(space_id);
    if (!space || !ms_table) return SGEMM_E_BADARG;
    if (strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    const int n = (int)space->configs.size();
    if (n == 0) return SGEMM_E_NOCONFIG;
    if (table_len != n) return SGEMM_E_BADARG;
    const SearchResult r = run_search(*space, strategy, budget, seed, params_from(opts),
                                      [&](int i) { return (double)ms_table[i]; });
    fill_result(*space, r, 0.0, out);
    if (visited)
        for (int i = 0; i < (int)r.visited.size() && i < visited_cap; ++i) visited[i] = r.visited[i];
    return r.evaluations;
}

int tune_ex(int M, int N, int K, int layout, float alpha, float beta, int strategy, int budget,
            unsigned long long seed, const tune_opts *opts, tune_result *out) {
    if (M <= 0 || N <= 0 || K <= 0 || M > kMaxSize || N > kMaxSize || K > kMaxSize || layout < 0 || layout > 3)
        return SGEMM_E_BADARG;
    if (strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    const Space *space = get_space(opts ? opts->space : SGEMM_SPACE_FULL);
    if (!space) return SGEMM_E_BADARG;
    if (space->configs.empty()) return SGEMM_E_NOCONFIG;
    const TimingRules rules = timing_rules_from(opts);
    const bool verify = !(opts && opts->verify_off);

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return SGEMM_E_NODEVICE;
    hipStream_t s;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        s = g_stream;
    }
    const auto wall0 = std::chrono::steady_clock::now();

    // ---- operands: the caller's, or library-owned synthetic ones -------------------------
    const int a_rows = (layout & 1) ? K : M, a_cols = (layout & 1) ? M : K;
    const int b_rows = (layout & 2) ? N : K, b_cols = (layout & 2) ? K : N;
    DeviceBuffer ownA, ownB, ownC, ownC0, ref, words;
    const float *A, *B, *C0 = nullptr;
    float *C;
    int lda, ldb, ldc;
    if (opts && opts->A) {
        if (!opts->B || !opts->C) return SGEMM_E_BADARG;
        A = opts->A; B = opts->B; C = opts->C; C0 = opts->C0;
        lda = opts->lda; ldb = opts->ldb; ldc = opts->ldc;
        if (lda < a_cols || ldb < b_cols || ldc < N) return SGEMM_E_BADARG;
        if (lda > kMaxLeadingDim || ldb > kMaxLeadingDim) return SGEMM_E_BADARG; // as in every GEMM call
        if (beta != 0.0f && !C0) return SGEMM_E_BADARG;
    } else {
        lda = a_cols; ldb = b_cols; ldc = N;
        if (ownA.alloc((size_t)a_rows * lda * 4) != hipSuccess || ownB.alloc((size_t)b_rows * ldb * 4) != hipSuccess ||
            ownC.alloc((size_t)M * ldc * 4) != hipSuccess)
            return SGEMM_E_LAUNCH;
        (void)sgemm_util::launch_fill_uniform(s, ownA.f(), a_rows, a_cols, lda, seed * 3 + 1);
        (void)sgemm_util::launch_fill_uniform(s, ownB.f(), b_rows, b_cols, ldb, seed * 3 + 2);
        A = ownA.f(); B = ownB.f(); C = ownC.f();
        if (beta != 0.0f) {
            if (ownC0.alloc((size_t)M * ldc * 4) != hipSuccess) return SGEMM_E_LAUNCH;
            (void)sgemm_util::launch_fill_uniform(s, ownC0.f(), M, N, ldc, seed * 3 + 3);
            C0 = ownC0.f();
        }
    }
    if (words.alloc(16) != hipSuccess) return SGEMM_E_LAUNCH;
    unsigned int *dwords = static_cast<unsigned int *>(words.p);

    // ---- reference result and tolerance, once per search ----------------------------------
    float abs_tol = 0.0f;
    const float rel_tol = 1e-6f;
    if (verify) {
        if (ref.alloc((size_t)M * N * 4) != hipSuccess) return SGEMM_E_LAUNCH;
        if (beta != 0.0f) (void)sgemm_util::launch_copy2d(s, ref.f(), N, C0, ldc, M, N);
        if (sgemm_util::launch_reference(s, M, N, K, alpha, A, lda, B, ldb, beta, ref.f(), N, layout) != hipSuccess)
            return SGEMM_E_LAUNCH;
        unsigned int bits[2] = {0, 0};
        (void)sgemm_util::launch_absmax(s, A, a_rows, a_cols, lda, dwords);
        (void)sgemm_util::launch_absmax(s, B, b_rows, b_cols, ldb, dwords + 1);
        if (hipMemcpyAsync(bits, dwords, 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return SGEMM_E_LAUNCH;
        float amax, bmax;
        std::memcpy(&amax, &bits[0], 4);
        std::memcpy(&bmax, &bits[1], 4);
        abs_tol = 1e-5f * (float)K * amax * bmax;
    }

    FILE *logf = (opts && opts->log_path) ? std::fopen(opts->log_path, "a") : nullptr;
    Event ev0, ev1;
    double best_ms = 0.0; // best so far, for the early cut
    double compile_ms_total = 0.0;
    int hip_failure = 0;
    const double flops = 2.0 * M * N * (double)K;

    auto evaluate = [&](int idx) -> double {
        const sgemm_config cfg = from_point(space->configs[idx]);
        const char *status = "ok";
        double ms = -1.0;
        sgemm_kernel_info info{};
        int samples = 0;
        do {
            if (hip_failure) { status = "skipped"; break; }
            const VariantKey key = resolve_variant(cfg, M, N, K, A, lda, B, ldb, C, ldc, layout, beta);
            std::shared_ptr<LoadedKernel> k;
            std::string log;
            const int rc = load_kernel(key, &k, &log);
            if (rc != SGEMM_OK) { status = rc == SGEMM_E_COMPILE ? "compile" : "load"; break; }
            info = k->info;
            compile_ms_total += info.compile_ms;
            if (info.scratch_bytes > 0) { status = "spill"; break; }
            if (info.lds_bytes > kLdsLimitBytes) { status = "lds"; break; }
            const Measured m = run_verify_time(
                s,
                // fresh C for the verified run, as every configuration gets fresh arguments
                // (beta == 0: C is not an input, so it is filled with NaN instead - an element the
                // variant fails to write must not pass for the previous variant's correct value)
                [&] {
                    if (beta != 0.0f) (void)sgemm_util::launch_copy2d(s, C, ldc, C0, ldc, M, N);
                    else if (verify) (void)sgemm_util::launch_fill_bits(s, C, M, N, ldc, 0x7fc00000u);
                },
                [&] { return launch_loaded(s, *k, key.cfg, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc) == SGEMM_OK; },
                verify ? std::function<int()>([&] {
                    unsigned int bits[2] = {0, 0};
                    (void)sgemm_util::launch_compare(s, C, ldc, ref.f(), N, M, N, abs_tol, rel_tol, dwords);
                    (void)hipMemcpyAsync(bits, dwords, 8, hipMemcpyDeviceToHost, s);
                    if (hipStreamSynchronize(s) != hipSuccess) return -1;
                    return bits[0] != 0 ? 1 : 0;
                }) : std::function<int()>(),
                rules, best_ms, ev0, ev1);
            status = m.status;
            samples = m.samples;
            if (m.device_failed) hip_failure = 1;
            if (std::strcmp(m.status, "ok") != 0) { if (std::strcmp(m.status, "ok-cut") == 0) ms = m.ms; break; }
            ms = m.ms;
            if (best_ms == 0.0 || ms < best_ms) best_ms = ms;
        } while (false);
        if (logf) {
            const Point p = space->configs[idx];
            std::fprintf(logf, "{\"M\":%d,\"N\":%d,\"K\":%d,\"layout\":%d,\"index\":%d,\"config\":[", M, N, K,
                         layout, idx);
            for (int d = 0; d < kDims; ++d) std::fprintf(logf, "%s%d", d ? "," : "", p[d]);
            std::fprintf(logf, "],\"status\":\"%s\",\"ms\":%.6g,\"gflops\":%.6g,\"samples\":%d,\"vgprs\":%d,"
                               "\"agprs\":%d,\"lds\":%d,\"scratch\":%d}\n",
                         status, ms, ms > 0 ? flops / (ms * 1e-3) * 1e-9 : 0.0, samples, info.vgprs,
                         info.agprs, info.lds_bytes, info.scratch_bytes);
            std::fflush(logf);
        }
        return ms;
    };

    StrategyParams sp = params_from(opts);
    if (opts && opts->warm_start > 0) {
        sgemm_config cached;
        std::lock_guard<std::mutex> lock(g_mu);
        select_config_locked(M, N, K, layout, &cached);
        sp.start_index = space->find(to_point(cached)); // -1 when it is not in this space
    }
    const SearchResult r = run_search(*space, strategy, budget, seed, sp, evaluate);
    if (logf) std::fclose(logf);
    (void)hipStreamSynchronize(s);
    fill_result(*space, r, flops, out);
    if (out) {
        out->compile_ms = (float)compile_ms_total;
        out->total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - wall0).count();
    }
    if (hip_failure) return SGEMM_E_LAUNCH;
    if (r.best_index < 0) return SGEMM_E_NOCONFIG;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        autoload_locked();
        auto it = g_tuned.find(ShapeKey{M, N, K, layout});
        if (it == g_tuned.end() || !(it->second.ms > 0) || r.best_cost < it->second.ms)
            g_tuned[ShapeKey{M, N, K, layout}] = Tuned{from_point(space->configs[r.best_index]), (float)r.best_cost};
        tuned_table_changed_locked();
    }
    return r.evaluations;
}

int tune(int M, int N, int K, int strategy, int budget) {
    return tune_ex(M, N, K, 0, 1.0f, 0.0f, strategy, budget, 0ull, nullptr, nullptr);
}

} // extern "C"
