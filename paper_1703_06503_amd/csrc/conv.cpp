// The second kernel family of the library: the tunable 2D convolution of the paper's first case
// study ("Case-study: 2D convolution").  Its search space, the dispatch of a call to a generated
// variant, and its tuning run, which uses the strategies, the timing rules and the verification
// of the GEMM tuner as they are.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <tuple>

#include "../../include/conv2d_tuned.h"
#include "internal.h"
#include "kernelgen.h"
#include "space.h"
#include "strategy.h"
#include "util_kernels.h"

using namespace sgemm;
using namespace sgemm::detail;

namespace {

constexpr int kConvDims = 8; // xwg ywg xwpt ywpt lmem vw pad unr

Point conv_to_point(const conv2d_config &c) {
    Point p{};
    p[0] = c.xwg; p[1] = c.ywg; p[2] = c.xwpt; p[3] = c.ywpt;
    p[4] = c.lmem; p[5] = c.vw; p[6] = c.pad; p[7] = c.unr;
    return p;
}

conv2d_config conv_from_point(const Point &p) {
    return conv2d_config{p[0], p[1], p[2], p[3], p[4], p[5], p[6], p[7]};
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

bool filter_ok(int Xf, int Yf) {
    return Xf >= 1 && Yf >= 1 && Xf <= CONV2D_MAX_FILTER && Yf <= CONV2D_MAX_FILTER;
}

int x_threads(const conv2d_config &c, int Xf) {
    return c.lmem == 2 ? c.xwg + ceil_div(Xf - 1, c.xwpt) : c.xwg;
}
int y_threads(const conv2d_config &c, int Yf) {
    return c.lmem == 2 ? c.ywg + ceil_div(Yf - 1, c.ywpt) : c.ywg;
}

int lds_bytes(const conv2d_config &c, int Xf, int Yf) {
    if (c.lmem == 0) return 0;
    if (c.lmem == 1) return 4 * (c.xwg * c.xwpt + Xf - 1 + c.pad) * (c.ywg * c.ywpt + Yf - 1);
    return 4 * (x_threads(c, Xf) * c.xwpt + c.pad) * (y_threads(c, Yf) * c.ywpt);
}

bool in_list(int v, std::initializer_list<int> l) {
    for (int x : l)
        if (x == v) return true;
    return false;
}

const char *violates(const conv2d_config &c, int Xf, int Yf) {
    if (!in_list(c.xwg, {8, 16, 32, 64}) || !in_list(c.ywg, {8, 16, 32, 64})) return "workgroup size not in {8,16,32,64}";
    if (!in_list(c.xwpt, {1, 2, 4, 8}) || !in_list(c.ywpt, {1, 2, 4, 8})) return "work per thread not in {1,2,4,8}";
    if (c.lmem < 0 || c.lmem > 2) return "LMEM not in {0,1,2}";
    if (!in_list(c.vw, {1, 2, 4, 8})) return "VW not in {1,2,4,8}";
    if (c.pad < 0 || c.pad > 1 || c.unr < 0 || c.unr > 1) return "PAD or UNR not in {0,1}";
    if (c.xwpt % c.vw) return "VW does not divide XWPT";
    if (c.lmem == 0 && c.pad) return "PAD without an LDS tile";
    if (x_threads(c, Xf) * y_threads(c, Yf) > kMaxThreads) return "more than 1024 threads";
    if (lds_bytes(c, Xf, Yf) > kLdsLimitBytes) return "LDS tile above 160 KiB";
    return nullptr;
}

std::mutex g_conv_mu;
std::map<std::pair<int, int>, std::unique_ptr<Space>> g_spaces;

const Space *conv_space(int Xf, int Yf) {
    if (!filter_ok(Xf, Yf)) return nullptr;
    std::lock_guard<std::mutex> lock(g_conv_mu);
    auto &slot = g_spaces[{Xf, Yf}];
    if (slot) return slot.get();
    auto s = std::make_unique<Space>();
    s->dims = kConvDims;
    s->values = {{8, 16, 32, 64}, {8, 16, 32, 64}, {1, 2, 4, 8}, {1, 2, 4, 8}, {0, 1, 2}, {1, 2, 4, 8}, {0, 1}, {0, 1}};
    s->raw = 1;
    for (auto &v : s->values) s->raw *= (long long)v.size();
    // the product in lexicographic order, first parameter slowest
    for (int a : s->values[0]) for (int b : s->values[1]) for (int c : s->values[2]) for (int d : s->values[3])
    for (int e : s->values[4]) for (int f : s->values[5]) for (int g : s->values[6]) for (int h : s->values[7]) {
        const conv2d_config cfg{a, b, c, d, e, f, g, h};
        if (violates(cfg, Xf, Yf)) continue;
        const Point p = conv_to_point(cfg);
        s->index.emplace(Space::key(p), (int)s->configs.size());
        s->configs.push_back(p);
    }
    slot = std::move(s);
    return slot.get();
}

// ---- variants ------------------------------------------------------------------------------
struct ConvVariant {
    conv2d_config cfg; // vw already narrowed to 1 for misaligned operands
    int Xf, Yf, edge;
    std::string macros() const {
        char buf[256];
        std::snprintf(buf, sizeof buf,
                      "-DXF=%d -DYF=%d -DXWG=%d -DYWG=%d -DXWPT=%d -DYWPT=%d -DLMEM=%d -DVW=%d -DPAD=%d "
                      "-DUNR=%d -DEDGE=%d",
                      Xf, Yf, cfg.xwg, cfg.ywg, cfg.xwpt, cfg.ywpt, cfg.lmem, cfg.vw, cfg.pad, cfg.unr, edge);
        return buf;
    }
};

std::map<std::string, std::shared_ptr<LoadedKernel>> g_loaded;
constexpr size_t kMaxLoaded = 512;

int get_loaded(const ConvVariant &v, std::shared_ptr<LoadedKernel> *out) {
    const std::string macros = v.macros();
    {
        std::lock_guard<std::mutex> lock(g_conv_mu);
        auto it = g_loaded.find(macros);
        if (it != g_loaded.end()) { *out = it->second; return SGEMM_OK; }
    }
    std::string log;
    std::shared_ptr<LoadedKernel> k;
    const int rc = load_kernel(conv_source(), macros, x_threads(v.cfg, v.Xf) * y_threads(v.cfg, v.Yf), &k, &log);
    if (rc != SGEMM_OK) { set_error(log); return rc; }
    std::lock_guard<std::mutex> lock(g_conv_mu);
    if (g_loaded.size() >= kMaxLoaded) {
        (void)hipDeviceSynchronize(); // no variant may still be running when its module goes away
        g_loaded.clear();
    }
    g_loaded[macros] = k;
    *out = std::move(k);
    return SGEMM_OK;
}

bool aligned_for(const void *p, int ld, int vw) {
    const int bytes = 4 * (vw > 4 ? 4 : vw); // 8-wide accesses are two of 4
    const int step = vw > 4 ? 4 : vw;
    return reinterpret_cast<uintptr_t>(p) % bytes == 0 && ld % step == 0;
}

ConvVariant resolve(const conv2d_config &cfg, int X, int Y, int Xf, int Yf, const float *A, int lda,
                    const float *B, int ldb) {
    ConvVariant v{cfg, Xf, Yf, 0};
    v.edge = (X % (cfg.xwg * cfg.xwpt) || Y % (cfg.ywg * cfg.ywpt)) ? 1 : 0;
    if (v.cfg.vw > 1 && !(aligned_for(A, lda, v.cfg.vw) && aligned_for(B, ldb, v.cfg.vw))) v.cfg.vw = 1;
    return v;
}

int check_args(int X, int Y, int Xf, int Yf, const float *F, const float *A, int lda, const float *B, int ldb) {
    if (X < 0 || Y < 0 || X > kMaxSize || Y > kMaxSize || !filter_ok(Xf, Yf)) {
        set_error("size negative or above 2^31 - 1025, or filter outside 1..31");
        return SGEMM_E_BADARG;
    }
    if (X == 0 || Y == 0) return SGEMM_OK;
    if (!F || !A || !B) { set_error("null operand"); return SGEMM_E_BADARG; }
    if (lda < X + Xf - 1 || ldb < X) { set_error("leading dimension too small (lda >= X + Xf - 1, ldb >= X)"); return SGEMM_E_BADARG; }
    return SGEMM_OK;
}

int launch(hipStream_t s, const LoadedKernel &k, const ConvVariant &v, int X, int Y, float w, const float *F,
           const float *A, int lda, float *B, int ldb) {
    const int tx = v.cfg.xwg * v.cfg.xwpt, ty = v.cfg.ywg * v.cfg.ywpt;
    const long long gx = ceil_div(X, tx), gy = ceil_div(Y, ty);
    if (gy > 65535) { set_error("more than 65535 workgroup rows"); return SGEMM_E_BADARG; }
    void *args[] = {&X, &Y, &w, &F, &A, &lda, &B, &ldb};
    const hipError_t e = hipModuleLaunchKernel(k.fn, (unsigned)gx, (unsigned)gy, 1, x_threads(v.cfg, v.Xf),
                                               y_threads(v.cfg, v.Yf), 1, 0, s, args, nullptr);
    if (e != hipSuccess) {
        set_error(std::string("hipModuleLaunchKernel: ") + hipGetErrorString(e) + " [" + v.macros() + "]");
        return SGEMM_E_LAUNCH;
    }
    return SGEMM_OK;
}

int run_config(hipStream_t s, const conv2d_config &cfg, int X, int Y, int Xf, int Yf, float w, const float *F,
               const float *A, int lda, float *B, int ldb) {
    const int rc = check_args(X, Y, Xf, Yf, F, A, lda, B, ldb);
    if (rc != SGEMM_OK) return rc;
    if (const char *why = violates(cfg, Xf, Yf)) { set_error(why); return SGEMM_E_INVALID; }
    if (X == 0 || Y == 0) return SGEMM_OK;
    const ConvVariant v = resolve(cfg, X, Y, Xf, Yf, A, lda, B, ldb);
    std::shared_ptr<LoadedKernel> k;
    const int lrc = get_loaded(v, &k);
    if (lrc != SGEMM_OK) return lrc;
    return launch(s, *k, v, X, Y, w, F, A, lda, B, ldb);
}

// ---- best configurations per problem ---------------------------------------------------------
struct TunedConv {
    conv2d_config cfg;
    float ms;
};
std::map<std::tuple<int, int, int, int>, TunedConv> g_tuned; // Xf, Yf, X, Y

// Built-in defaults: the winners of full searches on an 8192 x 4096 image with 3 x 3, 7 x 7 and
// 11 x 11 filters, each serving the filters nearest to it in number of taps.  All read their taps
// through the caches (LMEM = 0), so they are valid for every filter size.  Filters with more taps
// than were ever searched get a configuration whose filter loops stay loops: fully unrolled,
// their guarded builds run out of registers (measured on 13 x 13 to 31 x 31).
conv2d_config default_config(int Xf, int Yf) {
    const int taps = Xf * Yf;
    if (taps <= 16) return conv2d_config{64, 8, 4, 1, 0, 1, 0, 1};
    if (taps <= 81) return conv2d_config{32, 8, 8, 2, 0, 8, 0, 1};
    if (taps <= 121) return conv2d_config{32, 8, 4, 8, 0, 4, 0, 1};
    return conv2d_config{32, 8, 4, 4, 0, 4, 0, 0};
}

// 1 = exact entry, 0 = nearest image with the same filter or the default
int select_locked(int X, int Y, int Xf, int Yf, conv2d_config *out) {
    auto it = g_tuned.find({Xf, Yf, X, Y});
    if (it != g_tuned.end()) { *out = it->second.cfg; return 1; }
    double best = -1.0;
    *out = default_config(Xf, Yf);
    for (const auto &kv : g_tuned) {
        if (std::get<0>(kv.first) != Xf || std::get<1>(kv.first) != Yf) continue;
        const double d = std::fabs(std::log((double)std::max(1, X) / std::get<2>(kv.first))) +
                         std::fabs(std::log((double)std::max(1, Y) / std::get<3>(kv.first)));
        if (best < 0.0 || d < best) { best = d; *out = kv.second.cfg; }
    }
    return 0;
}

void fill_result(const Space &space, const SearchResult &r, int X, int Y, int Xf, int Yf, conv2d_tune_result *out) {
    if (!out) return;
    *out = conv2d_tune_result{};
    out->best_index = r.best_index;
    out->evaluations = r.evaluations;
    out->failed = r.failed;
    out->space_size = (int)space.configs.size();
    out->evals_to_best = r.evals_to_best;
    if (r.best_index >= 0) {
        out->best = conv_from_point(space.configs[r.best_index]);
        out->best_ms = (float)r.best_cost;
        const double sec = r.best_cost * 1e-3;
        out->best_gflops = (float)((1.0 + 2.0 * Xf * Yf) * X * (double)Y / sec * 1e-9);
        out->best_gbs = (float)(2.0 * X * (double)Y * 4.0 / sec * 1e-9);
    }
}

} // namespace

extern "C" {

int conv2d_space_size(int Xf, int Yf) {
    const Space *s = conv_space(Xf, Yf);
    return s ? (int)s->configs.size() : SGEMM_E_BADARG;
}

int conv2d_space_get(int Xf, int Yf, int index, conv2d_config *out) {
    const Space *s = conv_space(Xf, Yf);
    if (!s || !out || index < 0 || index >= (int)s->configs.size()) return SGEMM_E_BADARG;
    *out = conv_from_point(s->configs[index]);
    return SGEMM_OK;
}

int conv2d_space_find(int Xf, int Yf, const conv2d_config *cfg) {
    const Space *s = conv_space(Xf, Yf);
    if (!s || !cfg) return SGEMM_E_BADARG;
    const int i = s->find(conv_to_point(*cfg));
    return i >= 0 ? i : SGEMM_E_INVALID;
}

int conv2d_config_check(const conv2d_config *cfg, int Xf, int Yf) {
    if (!cfg || !filter_ok(Xf, Yf)) return SGEMM_E_BADARG;
    const char *why = violates(*cfg, Xf, Yf);
    if (why) set_error(why);
    return why ? SGEMM_E_INVALID : SGEMM_OK;
}

int conv2d_config_lds_bytes(const conv2d_config *cfg, int Xf, int Yf) {
    return (cfg && filter_ok(Xf, Yf)) ? lds_bytes(*cfg, Xf, Yf) : SGEMM_E_BADARG;
}

int conv2d_config_threads(const conv2d_config *cfg, int Xf, int Yf) {
    return (cfg && filter_ok(Xf, Yf)) ? x_threads(*cfg, Xf) * y_threads(*cfg, Yf) : SGEMM_E_BADARG;
}

int conv2d_kernel_compile(const conv2d_config *cfg, int Xf, int Yf, int edge, int vector, sgemm_kernel_info *info) {
    if (!cfg || !filter_ok(Xf, Yf)) return SGEMM_E_BADARG;
    if (const char *why = violates(*cfg, Xf, Yf)) { set_error(why); return SGEMM_E_INVALID; }
    ConvVariant v{*cfg, Xf, Yf, edge ? 1 : 0};
    if (!vector) v.cfg.vw = 1;
    CodeObject co;
    std::string log;
    const int rc = get_code_object(conv_source(), v.macros(), &co, &log);
    if (rc != SGEMM_OK) { set_error(log); return rc; }
    if (info) *info = co.info;
    return SGEMM_OK;
}

int conv2d_run_config(void *hip_stream, const conv2d_config *cfg, int X, int Y, int Xf, int Yf, float w,
                      const float *F, const float *A, int lda, float *B, int ldb) {
    if (!cfg) return SGEMM_E_BADARG;
    return run_config(static_cast<hipStream_t>(hip_stream), *cfg, X, Y, Xf, Yf, w, F, A, lda, B, ldb);
}

int conv2d_reference(void *hip_stream, int X, int Y, int Xf, int Yf, float w, const float *F, const float *A,
                     int lda, float *B, int ldb) {
    const int rc = check_args(X, Y, Xf, Yf, F, A, lda, B, ldb);
    if (rc != SGEMM_OK) return rc;
    const hipError_t e = sgemm_util::launch_conv2d_reference(static_cast<hipStream_t>(hip_stream), X, Y, Xf, Yf, w,
                                                             F, A, lda, B, ldb);
    if (e != hipSuccess) { set_error(std::string("reference kernel: ") + hipGetErrorString(e)); return SGEMM_E_LAUNCH; }
    return SGEMM_OK;
}

int conv2d_tuned(int X, int Y, int Xf, int Yf, float w, const float *F, const float *A, int lda, float *B,
                 int ldb) {
    const int rc = check_args(X, Y, Xf, Yf, F, A, lda, B, ldb);
    if (rc != SGEMM_OK) return rc;
    conv2d_config cfg;
    {
        std::lock_guard<std::mutex> lock(g_conv_mu);
        select_locked(X, Y, Xf, Yf, &cfg);
    }
    if (violates(cfg, Xf, Yf)) cfg = default_config(Xf, Yf);
    return run_config(library_stream(), cfg, X, Y, Xf, Yf, w, F, A, lda, B, ldb);
}

int conv2d_config_set(int X, int Y, int Xf, int Yf, const conv2d_config *cfg, float ms) {
    if (!cfg || X <= 0 || Y <= 0 || !filter_ok(Xf, Yf)) return SGEMM_E_BADARG;
    if (const char *why = violates(*cfg, Xf, Yf)) { set_error(why); return SGEMM_E_INVALID; }
    std::lock_guard<std::mutex> lock(g_conv_mu);
    g_tuned[{Xf, Yf, X, Y}] = TunedConv{*cfg, ms};
    return SGEMM_OK;
}

int conv2d_config_select(int X, int Y, int Xf, int Yf, conv2d_config *out) {
    if (!out || !filter_ok(Xf, Yf)) return SGEMM_E_BADARG;
    std::lock_guard<std::mutex> lock(g_conv_mu);
    return select_locked(X, Y, Xf, Yf, out);
}

int conv2d_cache_save(const char *path) {
    if (!path) return SGEMM_E_BADARG;
    FILE *f = std::fopen(path, "w");
    if (!f) { set_error(std::string("cannot write ") + path); return SGEMM_E_IO; }
    std::lock_guard<std::mutex> lock(g_conv_mu);
    std::fprintf(f, "# X Y Xf Yf ms XWG YWG XWPT YWPT LMEM VW PAD UNR\n");
    for (const auto &kv : g_tuned) {
        const conv2d_config &c = kv.second.cfg;
        std::fprintf(f, "%d %d %d %d %.6g %d %d %d %d %d %d %d %d\n", std::get<2>(kv.first), std::get<3>(kv.first),
                     std::get<0>(kv.first), std::get<1>(kv.first), kv.second.ms, c.xwg, c.ywg, c.xwpt, c.ywpt,
                     c.lmem, c.vw, c.pad, c.unr);
    }
    const int n = (int)g_tuned.size();
    return std::fclose(f) == 0 ? n : SGEMM_E_IO;
}

int conv2d_cache_load(const char *path) {
    if (!path) return SGEMM_E_BADARG;
    FILE *f = std::fopen(path, "r");
    if (!f) { set_error(std::string("cannot read ") + path); return SGEMM_E_IO; }
    char line[512];
    int n = 0;
    std::lock_guard<std::mutex> lock(g_conv_mu);
    while (std::fgets(line, sizeof line, f)) {
        int X, Y, Xf, Yf;
        float ms;
        conv2d_config c;
        if (line[0] == '#') continue;
        if (std::sscanf(line, "%d %d %d %d %f %d %d %d %d %d %d %d %d", &X, &Y, &Xf, &Yf, &ms, &c.xwg, &c.ywg,
                        &c.xwpt, &c.ywpt, &c.lmem, &c.vw, &c.pad, &c.unr) != 13)
            continue;
        if (X <= 0 || Y <= 0 || !filter_ok(Xf, Yf) || violates(c, Xf, Yf)) continue; // skip what this build cannot run
        auto it = g_tuned.find({Xf, Yf, X, Y});
        if (it == g_tuned.end() || !(it->second.ms > 0) || (ms > 0 && ms < it->second.ms)) g_tuned[{Xf, Yf, X, Y}] = TunedConv{c, ms};
        ++n;
    }
    std::fclose(f);
    return n;
}

int conv2d_cache_clear(void) {
    std::lock_guard<std::mutex> lock(g_conv_mu);
    g_tuned.clear();
    return SGEMM_OK;
}

int conv2d_tune_replay(int Xf, int Yf, const float *ms_table, int table_len, int strategy, int budget,
                       unsigned long long seed, const tune_opts *opts, int *visited, int visited_cap,
                       conv2d_tune_result *out) {
    const Space *space = conv_space(Xf, Yf);
    if (!space || !ms_table || strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    if (table_len != (int)space->configs.size()) return SGEMM_E_BADARG;
    const SearchResult r = run_search(*space, strategy, budget, seed, params_from(opts),
                                      [&](int i) { return (double)ms_table[i]; });
    fill_result(*space, r, 0, 0, Xf, Yf, out);
    if (visited)
        for (int i = 0; i < (int)r.visited.size() && i < visited_cap; ++i) visited[i] = r.visited[i];
    return r.evaluations;
}

int conv2d_tune(int X, int Y, int Xf, int Yf, float w, int strategy, int budget, unsigned long long seed,
                const tune_opts *opts, conv2d_tune_result *out) {
    if (X <= 0 || Y <= 0 || strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    const Space *space = conv_space(Xf, Yf);
    if (!space) return SGEMM_E_BADARG;
    if (space->configs.empty()) return SGEMM_E_NOCONFIG;
    const TimingRules rules = timing_rules_from(opts);
    const bool verify = !(opts && opts->verify_off);
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return SGEMM_E_NODEVICE;
    hipStream_t s = library_stream();
    const auto wall0 = std::chrono::steady_clock::now();

    // ---- library-owned seeded operands: image with halo, filter, output, reference output
    // rows of the image start at multiples of 64 bytes, so that every vector width can be used
    const int arows = Y + Yf - 1, lda = (X + Xf - 1 + 15) / 16 * 16, ldb = X;
    DeviceBuffer dA, dF, dB, ref, words;
    if (dA.alloc((size_t)arows * lda * 4) != hipSuccess || dF.alloc((size_t)Xf * Yf * 4) != hipSuccess ||
        dB.alloc((size_t)Y * ldb * 4) != hipSuccess || words.alloc(16) != hipSuccess)
        return SGEMM_E_LAUNCH;
    (void)sgemm_util::launch_fill_uniform(s, dA.f(), arows, lda, lda, seed * 3 + 1);
    (void)sgemm_util::launch_fill_uniform(s, dF.f(), Yf, Xf, Xf, seed * 3 + 2);
    unsigned int *dwords = static_cast<unsigned int *>(words.p);
    float abs_tol = 0.0f;
    const float rel_tol = 1e-6f;
    if (verify) {
        if (ref.alloc((size_t)Y * X * 4) != hipSuccess) return SGEMM_E_LAUNCH;
        if (sgemm_util::launch_conv2d_reference(s, X, Y, Xf, Yf, w, dF.f(), dA.f(), lda, ref.f(), X) != hipSuccess)
            return SGEMM_E_LAUNCH;
        unsigned int bits[2] = {0, 0};
        (void)sgemm_util::launch_absmax(s, dA.f(), arows, lda, lda, dwords);
        (void)sgemm_util::launch_absmax(s, dF.f(), Yf, Xf, Xf, dwords + 1);
        if (hipMemcpyAsync(bits, dwords, 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return SGEMM_E_LAUNCH;
        float amax, fmax;
        std::memcpy(&amax, &bits[0], 4);
        std::memcpy(&fmax, &bits[1], 4);
        abs_tol = 1e-5f * (float)(Xf * Yf) * std::fabs(w) * fmax * amax;
    }

    FILE *logf = (opts && opts->log_path) ? std::fopen(opts->log_path, "a") : nullptr;
    Event ev0, ev1;
    double best_ms = 0.0, compile_ms_total = 0.0;
    int hip_failure = 0;
    const double flops = (1.0 + 2.0 * Xf * Yf) * X * (double)Y;

    auto evaluate = [&](int idx) -> double {
        const conv2d_config cfg = conv_from_point(space->configs[idx]);
        const char *status = "ok";
        double ms = -1.0;
        sgemm_kernel_info info{};
        int samples = 0;
        do {
            if (hip_failure) { status = "skipped"; break; }
            const ConvVariant v = resolve(cfg, X, Y, Xf, Yf, dA.f(), lda, dB.f(), ldb);
            std::shared_ptr<LoadedKernel> k;
            std::string log;
            const int rc = load_kernel(conv_source(), v.macros(), x_threads(cfg, Xf) * y_threads(cfg, Yf), &k, &log);
            if (rc != SGEMM_OK) { status = rc == SGEMM_E_COMPILE ? "compile" : "load"; break; }
            info = k->info;
            compile_ms_total += info.compile_ms;
            if (info.scratch_bytes > 0) { status = "spill"; break; }
            if (info.lds_bytes > kLdsLimitBytes) { status = "lds"; break; }
            const Measured m = run_verify_time(
                s,
                // fresh output for the verified run: a NaN in every element, so that an output the
                // variant fails to write cannot pass for the previous variant's correct value
                [&] { if (verify) (void)sgemm_util::launch_fill_bits(s, dB.f(), Y, X, ldb, 0x7fc00000u); },
                [&] { return launch(s, *k, v, X, Y, w, dF.f(), dA.f(), lda, dB.f(), ldb) == SGEMM_OK; },
                verify ? std::function<int()>([&] {
                    unsigned int bits[2] = {0, 0};
                    (void)sgemm_util::launch_compare(s, dB.f(), ldb, ref.f(), X, Y, X, abs_tol, rel_tol, dwords);
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
            std::fprintf(logf, "{\"X\":%d,\"Y\":%d,\"Xf\":%d,\"Yf\":%d,\"index\":%d,\"config\":[", X, Y, Xf, Yf, idx);
            for (int d = 0; d < kConvDims; ++d) std::fprintf(logf, "%s%d", d ? "," : "", p[d]);
            std::fprintf(logf, "],\"status\":\"%s\",\"ms\":%.6g,\"gflops\":%.6g,\"samples\":%d,\"vgprs\":%d,"
                               "\"lds\":%d,\"scratch\":%d}\n",
                         status, ms, ms > 0 ? flops / (ms * 1e-3) * 1e-9 : 0.0, samples, info.vgprs,
                         info.lds_bytes, info.scratch_bytes);
            std::fflush(logf);
        }
        return ms;
    };

    const SearchResult r = run_search(*space, strategy, budget, seed, params_from(opts), evaluate);
    if (logf) std::fclose(logf);
    (void)hipStreamSynchronize(s);
    fill_result(*space, r, X, Y, Xf, Yf, out);
    if (out) {
        out->compile_ms = (float)compile_ms_total;
        out->total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - wall0).count();
    }
    if (hip_failure) return SGEMM_E_LAUNCH;
    if (r.best_index < 0) return SGEMM_E_NOCONFIG;
    {
        std::lock_guard<std::mutex> lock(g_conv_mu);
        auto it = g_tuned.find({Xf, Yf, X, Y});
        if (it == g_tuned.end() || !(it->second.ms > 0) || r.best_cost < it->second.ms)
            g_tuned[{Xf, Yf, X, Y}] = TunedConv{conv_from_point(space->configs[r.best_index]), (float)r.best_cost};
    }
    return r.evaluations;
}

} // extern "C"
