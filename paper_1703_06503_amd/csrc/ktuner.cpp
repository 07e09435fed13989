// The generic tuner: the paper's user-facing method (section "CLTune: an auto-tuner for OpenCL
// kernels": add a kernel, name parameters, modify the thread counts by them, constrain, verify
// against a reference kernel, search) for any HIP kernel, on the library's kernel generator,
// strategies and timing rules.
#include <hip/hip_runtime_api.h>

#include <cctype>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <string>
#include <vector>

#include "../../include/kernel_tuner.h"
#include "internal.h"
#include "kernelgen.h"
#include "space.h"
#include "strategy.h"
#include "util_kernels.h"

using namespace sgemm;
using namespace sgemm::detail;

namespace {

struct Modifier {
    bool global, multiply;
    int param[3]; // index of the parameter per dimension, -1 = none
};

struct Constraint {
    ktuner_constraint_fn fn;
    std::vector<int> params;
    void *user;
};

struct Argument {
    enum Kind { Input, Output, Int, Float } kind;
    std::vector<char> host; // buffers: the caller's data
    int i = 0;
    float f = 0.0f;
    DeviceBuffer pristine, work, ref; // device copies (ref: outputs only)
    void *dev_ptr = nullptr;          // what the kernel receives (work.p)
};

} // namespace

struct ktuner {
    std::string source, entry, ref_source, ref_entry;
    int global[3], local[3], ref_global[3], ref_local[3];
    bool has_reference = false;
    std::vector<std::string> names;
    std::vector<Modifier> modifiers;
    std::vector<Constraint> constraints;
    std::vector<std::unique_ptr<Argument>> args;
    float abs_tol = -1.0f, rel_tol = -1.0f;
    Space space;
    bool space_built = false;
    std::vector<float> times; // per configuration, after a tuning run
    int best_index = -1;
};

namespace {

bool is_identifier(const char *s) {
    if (!s || !*s || !(std::isalpha((unsigned char)*s) || *s == '_')) return false;
    for (const char *p = s; *p; ++p)
        if (!(std::isalnum((unsigned char)*p) || *p == '_')) return false;
    return true;
}

int param_index(const ktuner *t, const char *name) {
    for (size_t i = 0; i < t->names.size(); ++i)
        if (t->names[i] == name) return (int)i;
    return -1;
}

// Thread counts of one configuration; false when a division leaves a remainder, the global
// size is not a multiple of the local size, or a device limit is exceeded.
bool launch_shape(const ktuner *t, const Point &p, int grid[3], int block[3]) {
    long long g[3] = {t->global[0], t->global[1], t->global[2]};
    long long l[3] = {t->local[0], t->local[1], t->local[2]};
    for (const Modifier &m : t->modifiers) {
        long long *v = m.global ? g : l;
        for (int d = 0; d < 3; ++d) {
            if (m.param[d] < 0) continue;
            const int by = p[m.param[d]];
            if (by <= 0) return false;
            if (m.multiply) v[d] *= by;
            else if (v[d] % by) return false;
            else v[d] /= by;
        }
    }
    long long threads = 1;
    for (int d = 0; d < 3; ++d) {
        if (g[d] <= 0 || l[d] <= 0 || g[d] % l[d]) return false;
        threads *= l[d];
        if (g[d] / l[d] > (d == 0 ? 2147483647ll : 65535ll)) return false;
        grid[d] = (int)(g[d] / l[d]);
        block[d] = (int)l[d];
    }
    return threads <= kMaxThreads;
}

std::string macros_of(const ktuner *t, const Point &p) {
    std::string m;
    for (size_t d = 0; d < t->names.size(); ++d) {
        if (d) m += ' ';
        m += "-D" + t->names[d] + "=" + std::to_string(p[d]);
    }
    return m;
}

KernelSource source_of(const ktuner *t) {
    return KernelSource{t->source.data(), t->source.data() + t->source.size(), "tuned_kernel.hip",
                        t->entry.c_str()};
}

int add_modifier(ktuner *t, bool global, bool multiply, const char *const names[3]) {
    if (!t || !names) return SGEMM_E_BADARG;
    Modifier m{global, multiply, {-1, -1, -1}};
    for (int d = 0; d < 3; ++d) {
        if (!names[d]) continue;
        m.param[d] = param_index(t, names[d]);
        if (m.param[d] < 0) { set_error(std::string("unknown parameter ") + names[d]); return SGEMM_E_BADARG; }
    }
    t->modifiers.push_back(m);
    t->space_built = false;
    return SGEMM_OK;
}

int add_buffer(ktuner *t, Argument::Kind kind, const void *host, size_t bytes) {
    if (!t || !host || bytes == 0) return SGEMM_E_BADARG;
    if (kind == Argument::Output && (bytes % 4 || bytes / 4 > 0x7fffffffull)) {
        set_error("output arguments are float arrays of fewer than 2^31 elements");
        return SGEMM_E_BADARG;
    }
    auto a = std::make_unique<Argument>();
    a->kind = kind;
    a->host.assign(static_cast<const char *>(host), static_cast<const char *>(host) + bytes);
    t->args.push_back(std::move(a));
    return SGEMM_OK;
}

} // namespace

extern "C" {

ktuner *ktuner_create(const char *source, const char *entry, const int global[3], const int local[3]) {
    if (!source || !is_identifier(entry) || !global || !local) return nullptr;
    for (int d = 0; d < 3; ++d)
        if (global[d] <= 0 || local[d] <= 0) return nullptr;
    auto *t = new ktuner();
    t->source = source;
    t->entry = entry;
    std::memcpy(t->global, global, sizeof t->global);
    std::memcpy(t->local, local, sizeof t->local);
    return t;
}

void ktuner_destroy(ktuner *t) { delete t; }

int ktuner_add_parameter(ktuner *t, const char *name, const int *values, int n) {
    if (!t || !is_identifier(name) || !values || n <= 0) return SGEMM_E_BADARG;
    if ((int)t->names.size() >= KTUNER_MAX_PARAMETERS) { set_error("too many parameters"); return SGEMM_E_BADARG; }
    if (param_index(t, name) >= 0) { set_error(std::string("parameter named twice: ") + name); return SGEMM_E_BADARG; }
    t->names.push_back(name);
    t->space.values.emplace_back(values, values + n);
    t->space_built = false;
    return SGEMM_OK;
}

int ktuner_mul_global_size(ktuner *t, const char *const names[3]) { return add_modifier(t, true, true, names); }
int ktuner_div_global_size(ktuner *t, const char *const names[3]) { return add_modifier(t, true, false, names); }
int ktuner_mul_local_size(ktuner *t, const char *const names[3]) { return add_modifier(t, false, true, names); }
int ktuner_div_local_size(ktuner *t, const char *const names[3]) { return add_modifier(t, false, false, names); }

int ktuner_add_constraint(ktuner *t, ktuner_constraint_fn fn, const char *const *names, int n, void *user) {
    if (!t || !fn || !names || n <= 0) return SGEMM_E_BADARG;
    Constraint c{fn, {}, user};
    for (int i = 0; i < n; ++i) {
        const int p = names[i] ? param_index(t, names[i]) : -1;
        if (p < 0) { set_error("constraint on an unknown parameter"); return SGEMM_E_BADARG; }
        c.params.push_back(p);
    }
    t->constraints.push_back(std::move(c));
    t->space_built = false;
    return SGEMM_OK;
}

int ktuner_add_argument_input(ktuner *t, const void *host, size_t bytes) { return add_buffer(t, Argument::Input, host, bytes); }
int ktuner_add_argument_output(ktuner *t, const void *host, size_t bytes) { return add_buffer(t, Argument::Output, host, bytes); }

int ktuner_add_argument_int(ktuner *t, int value) {
    if (!t) return SGEMM_E_BADARG;
    auto a = std::make_unique<Argument>();
    a->kind = Argument::Int;
    a->i = value;
    t->args.push_back(std::move(a));
    return SGEMM_OK;
}

int ktuner_add_argument_float(ktuner *t, float value) {
    if (!t) return SGEMM_E_BADARG;
    auto a = std::make_unique<Argument>();
    a->kind = Argument::Float;
    a->f = value;
    t->args.push_back(std::move(a));
    return SGEMM_OK;
}

int ktuner_set_reference(ktuner *t, const char *source, const char *entry, const int global[3], const int local[3]) {
    if (!t || !source || !is_identifier(entry) || !global || !local) return SGEMM_E_BADARG;
    long long threads = 1;
    for (int d = 0; d < 3; ++d) {
        if (global[d] <= 0 || local[d] <= 0 || global[d] % local[d]) return SGEMM_E_BADARG;
        threads *= local[d];
    }
    if (threads > kMaxThreads) return SGEMM_E_BADARG;
    t->ref_source = source;
    t->ref_entry = entry;
    std::memcpy(t->ref_global, global, sizeof t->ref_global);
    std::memcpy(t->ref_local, local, sizeof t->ref_local);
    t->has_reference = true;
    return SGEMM_OK;
}

int ktuner_set_tolerance(ktuner *t, float abs_tol, float rel_tol) {
    if (!t) return SGEMM_E_BADARG;
    t->abs_tol = abs_tol;
    t->rel_tol = rel_tol;
    return SGEMM_OK;
}

} // extern "C"

namespace {

// The product of the value lists in lexicographic order, pruned by the caller's constraints
// and by the thread-count rules.
void enumerate(ktuner *t) {
    if (t->space_built) return;
    Space &s = t->space;
    s.dims = (int)t->names.size();
    s.configs.clear();
    s.index.clear();
    s.raw = 1;
    for (auto &v : s.values) s.raw *= (long long)v.size();
    t->space_built = true;
    t->times.clear();
    t->best_index = -1;
    if (s.dims == 0) return;
    std::vector<size_t> it(s.dims, 0);
    std::vector<int> cvals;
    for (;;) {
        Point p{};
        for (int d = 0; d < s.dims; ++d) p[d] = s.values[d][it[d]];
        bool ok = true;
        for (const Constraint &c : t->constraints) {
            cvals.clear();
            for (int q : c.params) cvals.push_back(p[q]);
            if (!c.fn(cvals.data(), c.user)) { ok = false; break; }
        }
        int grid[3], block[3];
        if (ok && launch_shape(t, p, grid, block)) {
            s.index.emplace(Space::key(p), (int)s.configs.size());
            s.configs.push_back(p);
        }
        int d = s.dims - 1;
        while (d >= 0 && ++it[d] == s.values[d].size()) it[d--] = 0;
        if (d < 0) break;
    }
}

} // namespace

extern "C" {

int ktuner_space_size(ktuner *t) {
    if (!t) return SGEMM_E_BADARG;
    enumerate(t);
    return (int)t->space.configs.size();
}

int ktuner_space_get(ktuner *t, int index, int *values) {
    if (!t || !values) return SGEMM_E_BADARG;
    enumerate(t);
    if (index < 0 || index >= (int)t->space.configs.size()) return SGEMM_E_BADARG;
    for (int d = 0; d < t->space.dims; ++d) values[d] = t->space.configs[index][d];
    return SGEMM_OK;
}

int ktuner_compile(ktuner *t, int index, sgemm_kernel_info *info) {
    if (!t) return SGEMM_E_BADARG;
    enumerate(t);
    if (index < 0 || index >= (int)t->space.configs.size()) return SGEMM_E_BADARG;
    CodeObject co;
    std::string log;
    const int rc = get_code_object(source_of(t), macros_of(t, t->space.configs[index]), &co, &log);
    if (rc != SGEMM_OK) set_error(log);
    if (info) *info = co.info;
    return rc;
}

int ktuner_launch_shape(ktuner *t, int index, int grid[3], int block[3]) {
    if (!t || !grid || !block) return SGEMM_E_BADARG;
    enumerate(t);
    if (index < 0 || index >= (int)t->space.configs.size()) return SGEMM_E_BADARG;
    return launch_shape(t, t->space.configs[index], grid, block) ? SGEMM_OK : SGEMM_E_INVALID;
}

float ktuner_time_of(ktuner *t, int index) {
    if (!t || index < 0 || index >= (int)t->times.size()) return 0.0f;
    return t->times[index];
}

int ktuner_read_output(ktuner *t, int which, void *host, size_t bytes) {
    if (!t || !host || which < 0) return SGEMM_E_BADARG;
    for (auto &a : t->args) {
        if (a->kind != Argument::Output) continue;
        if (which-- > 0) continue;
        if (!a->work.p || bytes > a->host.size()) return SGEMM_E_BADARG;
        return hipMemcpy(host, a->work.p, bytes, hipMemcpyDeviceToHost) == hipSuccess ? SGEMM_OK : SGEMM_E_LAUNCH;
    }
    return SGEMM_E_BADARG;
}

int ktuner_tune(ktuner *t, int strategy, int budget, unsigned long long seed, const tune_opts *opts,
                ktuner_result *out) {
    if (!t || strategy < 0 || strategy > 3) return SGEMM_E_BADARG;
    enumerate(t);
    const Space &space = t->space;
    if (space.configs.empty()) return SGEMM_E_NOCONFIG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return SGEMM_E_NODEVICE;
    hipStream_t s = library_stream();
    const TimingRules rules = timing_rules_from(opts);
    const bool verify = t->has_reference && !(opts && opts->verify_off);
    const auto wall0 = std::chrono::steady_clock::now();

    // ---- device copies of the arguments -------------------------------------------------
    std::vector<void *> argv;
    for (auto &a : t->args) {
        if (a->kind == Argument::Int) { argv.push_back(&a->i); continue; }
        if (a->kind == Argument::Float) { argv.push_back(&a->f); continue; }
        const size_t n = a->host.size();
        if (!a->pristine.p && a->pristine.alloc(n) != hipSuccess) return SGEMM_E_LAUNCH;
        if (!a->work.p && a->work.alloc(n) != hipSuccess) return SGEMM_E_LAUNCH;
        if (hipMemcpy(a->pristine.p, a->host.data(), n, hipMemcpyHostToDevice) != hipSuccess) return SGEMM_E_LAUNCH;
        a->dev_ptr = a->work.p;
        argv.push_back(&a->dev_ptr);
    }
    auto refresh = [&]() {
        for (auto &a : t->args)
            if (a->kind == Argument::Input || a->kind == Argument::Output)
                (void)hipMemcpyAsync(a->work.p, a->pristine.p, a->host.size(), hipMemcpyDeviceToDevice, s);
    };

    // ---- the reference kernel's outputs, once ---------------------------------------------
    DeviceBuffer words;
    if (words.alloc(16) != hipSuccess) return SGEMM_E_LAUNCH;
    unsigned int *dwords = static_cast<unsigned int *>(words.p);
    std::vector<float> abs_tols;
    if (verify) {
        std::shared_ptr<LoadedKernel> rk;
        std::string log;
        const KernelSource rsrc{t->ref_source.data(), t->ref_source.data() + t->ref_source.size(),
                                "reference_kernel.hip", t->ref_entry.c_str()};
        const int rc = load_kernel(rsrc, "", t->ref_local[0] * t->ref_local[1] * t->ref_local[2], &rk, &log);
        if (rc != SGEMM_OK) { set_error("reference kernel: " + log); return rc; }
        refresh();
        if (hipModuleLaunchKernel(rk->fn, t->ref_global[0] / t->ref_local[0], t->ref_global[1] / t->ref_local[1],
                                  t->ref_global[2] / t->ref_local[2], t->ref_local[0], t->ref_local[1],
                                  t->ref_local[2], 0, s, argv.data(), nullptr) != hipSuccess) {
            set_error("launch of the reference kernel failed");
            return SGEMM_E_LAUNCH;
        }
        for (auto &a : t->args) {
            if (a->kind != Argument::Output) continue;
            const size_t n = a->host.size();
            if (!a->ref.p && a->ref.alloc(n) != hipSuccess) return SGEMM_E_LAUNCH;
            (void)hipMemcpyAsync(a->ref.p, a->work.p, n, hipMemcpyDeviceToDevice, s);
            unsigned int bits = 0;
            (void)sgemm_util::launch_absmax(s, a->ref.f(), 1, (int)(n / 4), (int)(n / 4), dwords);
            if (hipMemcpyAsync(&bits, dwords, 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess) {
                set_error("the reference kernel failed on the device");
                return SGEMM_E_LAUNCH;
            }
            float refmax;
            std::memcpy(&refmax, &bits, 4);
            abs_tols.push_back(t->abs_tol >= 0.0f ? t->abs_tol : 1e-6f * refmax);
        }
        (void)hipStreamSynchronize(s); // before rk, and with it the reference kernel's module, goes away
    }
    const float rel_tol = t->rel_tol >= 0.0f ? t->rel_tol : 1e-5f;

    FILE *logf = (opts && opts->log_path) ? std::fopen(opts->log_path, "a") : nullptr;
    Event ev0, ev1;
    double best_ms = 0.0, compile_ms_total = 0.0;
    int hip_failure = 0, failed_verify = 0;
    t->times.assign(space.configs.size(), 0.0f);
    const KernelSource src = source_of(t);

    auto evaluate = [&](int idx) -> double {
        const Point &p = space.configs[idx];
        const char *status = "ok";
        double ms = -1.0;
        sgemm_kernel_info info{};
        int samples = 0;
        do {
            if (hip_failure) { status = "skipped"; break; }
            int grid[3], block[3];
            if (!launch_shape(t, p, grid, block)) { status = "shape"; break; }
            std::shared_ptr<LoadedKernel> k;
            std::string log;
            const int rc = load_kernel(src, macros_of(t, p), block[0] * block[1] * block[2], &k, &log);
            if (rc != SGEMM_OK) { status = rc == SGEMM_E_COMPILE ? "compile" : "load"; set_error(log); break; }
            info = k->info;
            compile_ms_total += info.compile_ms;
            if (info.lds_bytes > kLdsLimitBytes) { status = "lds"; break; }
            const Measured m = run_verify_time(
                s, refresh, // a fresh copy of every argument for the verified run
                [&] {
                    return hipModuleLaunchKernel(k->fn, grid[0], grid[1], grid[2], block[0], block[1], block[2], 0, s,
                                                 argv.data(), nullptr) == hipSuccess;
                },
                verify ? std::function<int()>([&] {
                    bool differs = false;
                    size_t o = 0;
                    for (auto &a : t->args) {
                        if (a->kind != Argument::Output) continue;
                        const int n = (int)(a->host.size() / 4);
                        unsigned int bits[2] = {0, 0};
                        (void)sgemm_util::launch_compare(s, a->work.f(), n, a->ref.f(), n, 1, n, abs_tols[o++], rel_tol, dwords);
                        (void)hipMemcpyAsync(bits, dwords, 8, hipMemcpyDeviceToHost, s);
                        if (hipStreamSynchronize(s) != hipSuccess) return -1;
                        if (bits[0] != 0) differs = true;
                    }
                    return differs ? 1 : 0;
                }) : std::function<int()>(),
                rules, best_ms, ev0, ev1);
            status = m.status;
            samples = m.samples;
            if (m.device_failed) hip_failure = 1;
            if (std::strcmp(m.status, "verify") == 0) ++failed_verify;
            if (std::strcmp(m.status, "ok") != 0) { if (std::strcmp(m.status, "ok-cut") == 0) ms = m.ms; break; }
            ms = m.ms;
            if (best_ms == 0.0 || ms < best_ms) best_ms = ms;
        } while (false);
        t->times[idx] = (float)ms;
        if (logf) {
            std::fprintf(logf, "{\"index\":%d,\"config\":{", idx);
            for (int d = 0; d < space.dims; ++d) std::fprintf(logf, "%s\"%s\":%d", d ? "," : "", t->names[d].c_str(), p[d]);
            std::fprintf(logf, "},\"status\":\"%s\",\"ms\":%.6g,\"samples\":%d,\"vgprs\":%d,\"lds\":%d,\"scratch\":%d}\n",
                         status, ms, samples, info.vgprs, info.lds_bytes, info.scratch_bytes);
            std::fflush(logf);
        }
        return ms;
    };

    const SearchResult r = run_search(space, strategy, budget, seed, params_from(opts), evaluate);
    if (logf) std::fclose(logf);
    t->best_index = r.best_index;
    // leave the outputs as the best configuration computes them
    if (r.best_index >= 0 && !hip_failure) {
        int grid[3], block[3];
        std::shared_ptr<LoadedKernel> k;
        std::string log;
        const Point &p = space.configs[r.best_index];
        if (launch_shape(t, p, grid, block) &&
            load_kernel(src, macros_of(t, p), block[0] * block[1] * block[2], &k, &log) == SGEMM_OK) {
            refresh();
            (void)hipModuleLaunchKernel(k->fn, grid[0], grid[1], grid[2], block[0], block[1], block[2], 0, s,
                                        argv.data(), nullptr);
            (void)hipStreamSynchronize(s); // before k, and with it the module, goes away
        }
    }
    (void)hipStreamSynchronize(s);
    if (out) {
        *out = ktuner_result{};
        out->best_index = r.best_index;
        out->best_ms = r.best_index >= 0 ? (float)r.best_cost : 0.0f;
        out->evaluations = r.evaluations;
        out->failed = r.failed;
        out->failed_verify = failed_verify;
        out->space_size = (int)space.configs.size();
        out->evals_to_best = r.evals_to_best;
        out->compile_ms = (float)compile_ms_total;
        out->total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - wall0).count();
    }
    if (hip_failure) return SGEMM_E_LAUNCH;
    if (r.best_index < 0) return SGEMM_E_NOCONFIG;
    return r.evaluations;
}

} // extern "C"
