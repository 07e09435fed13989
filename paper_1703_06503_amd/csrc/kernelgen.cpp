#include "kernelgen.h"
#include "space.h"

#include <dlfcn.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

// The kernel source travels inside the library: assembled in from the .inc file at build time.
__asm__(".section .rodata\n"
        ".global sgemm_kernel_source_begin\n"
        "sgemm_kernel_source_begin:\n"
        ".incbin \"" SGEMM_KERNEL_SOURCE_PATH "\"\n"
        ".global sgemm_kernel_source_end\n"
        "sgemm_kernel_source_end:\n"
        ".byte 0\n"
        ".previous\n");
extern "C" const char sgemm_kernel_source_begin[];
extern "C" const char sgemm_kernel_source_end[];
__asm__(".section .rodata\n"
        ".global conv_kernel_source_begin\n"
        "conv_kernel_source_begin:\n"
        ".incbin \"" CONV_KERNEL_SOURCE_PATH "\"\n"
        ".global conv_kernel_source_end\n"
        "conv_kernel_source_end:\n"
        ".byte 0\n"
        ".previous\n");
extern "C" const char conv_kernel_source_begin[];
extern "C" const char conv_kernel_source_end[];

namespace sgemm {

namespace {

std::mutex g_mu;
std::string g_cache_dir;

uint64_t fnv1a(const void *data, size_t n, uint64_t h = 1469598103934665603ull) {
    const unsigned char *p = static_cast<const unsigned char *>(data);
    for (size_t i = 0; i < n; ++i) { h ^= p[i]; h *= 1099511628211ull; }
    return h;
}

std::string default_cache_dir() {
    if (const char *env = std::getenv("SGEMM_TUNED_CACHE_DIR"))
        if (*env) return env; // an empty value counts as unset
    Dl_info info;
    if (dladdr((const void *)&default_cache_dir, &info) && info.dli_fname) {
        std::string p = info.dli_fname;
        const size_t slash = p.find_last_of('/');
        p = (slash == std::string::npos) ? "." : p.substr(0, slash);
        return p + "/kcache";
    }
    return "./kcache";
}

bool read_file(const std::string &path, std::vector<char> *out) {
    FILE *f = std::fopen(path.c_str(), "rb");
    if (!f) return false;
    std::fseek(f, 0, SEEK_END);
    const long n = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    out->resize(n > 0 ? (size_t)n : 0);
    const bool ok = n > 0 && std::fread(out->data(), 1, (size_t)n, f) == (size_t)n;
    std::fclose(f);
    return ok;
}

void write_file_atomic(const std::string &path, const std::vector<char> &data) {
    char tmp[64];
    std::snprintf(tmp, sizeof tmp, ".tmp.%d", (int)getpid());
    const std::string t = path + tmp;
    FILE *f = std::fopen(t.c_str(), "wb");
    if (!f) return;
    const bool ok = std::fwrite(data.data(), 1, data.size(), f) == data.size();
    std::fclose(f);
    if (ok) std::rename(t.c_str(), path.c_str());
    else std::remove(t.c_str());
}

const char *const kCompilerFlags[] = {
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    // packed-FP32 instructions are kept out of every variant
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
};

// Finds msgpack key `name` in the metadata and decodes the unsigned integer that follows.
bool find_uint(const std::vector<char> &img, const char *name, long long *value) {
    const size_t n = std::strlen(name);
    const unsigned char *b = reinterpret_cast<const unsigned char *>(img.data());
    for (size_t i = 0; i + n + 1 < img.size(); ++i) {
        if (std::memcmp(b + i, name, n) != 0) continue;
        const unsigned char *p = b + i + n;
        const size_t left = img.size() - (i + n);
        if (p[0] <= 0x7f) { *value = p[0]; return true; }
        if (p[0] == 0xcc && left >= 2) { *value = p[1]; return true; }
        if (p[0] == 0xcd && left >= 3) { *value = (p[1] << 8) | p[2]; return true; }
        if (p[0] == 0xce && left >= 5) {
            *value = ((long long)p[1] << 24) | (p[2] << 16) | (p[3] << 8) | p[4];
            return true;
        }
    }
    return false;
}

// Folds the identity of the compiler in use into a cache key: hipRTC's version and the path
// and size of the hipRTC library this process resolved (two ROCm installs report one version).
uint64_t compiler_identity(uint64_t h) {
    static std::once_flag once;
    static std::string ident;
    std::call_once(once, [] {
        int major = 0, minor = 0;
        hiprtcVersion(&major, &minor);
        ident = std::to_string(major) + "." + std::to_string(minor);
        Dl_info info;
        if (dladdr((const void *)&hiprtcCompileProgram, &info) && info.dli_fname) {
            ident += std::string(":") + info.dli_fname;
            struct stat st;
            if (stat(info.dli_fname, &st) == 0) ident += ":" + std::to_string((long long)st.st_size);
        }
    });
    return fnv1a(ident.data(), ident.size(), h);
}

} // namespace

std::string VariantKey::macros() const {
    char buf[512];
    std::snprintf(buf, sizeof buf,
                  "-DMWG=%d -DNWG=%d -DKWG=%d -DMDIMC=%d -DNDIMC=%d -DVWM=%d -DVWN=%d -DSA=%d "
                  "-DSB=%d -DPAD=%d -DKWI=%d -DMFMA=%d -DGRP=%d -DNS=%d -DTRA=%d -DTRB=%d -DEDGE=%d -DSPLITK=%d",
                  cfg.mwg, cfg.nwg, cfg.kwg, cfg.mdimc, cfg.ndimc, cfg.vwm, cfg.vwn, cfg.sa, cfg.sb,
                  cfg.pad, cfg.kwi, cfg.mfma, cfg.grp, cfg.ns > 0 ? cfg.ns : 2, layout & 1,
                  (layout >> 1) & 1, edge ? 1 : 0, splitk ? 1 : 0);
    std::string out = buf;
    // only where it differs from the source's default: builds without it keep their cache names
    if (cfg.ksw > 1) out += " -DKSW=" + std::to_string(cfg.ksw);
    if (cpf) out += " -DCPF=1";
    return out;
}

void set_cache_dir(const std::string &path) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_cache_dir = path;
}

std::string cache_dir() {
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_cache_dir.empty()) g_cache_dir = default_cache_dir();
    return g_cache_dir;
}

void read_code_object_info(const std::vector<char> &image, sgemm_kernel_info *info) {
    long long v;
    info->code_bytes = (int)image.size();
    if (find_uint(image, ".vgpr_count", &v)) info->vgprs = (int)v;
    if (find_uint(image, ".agpr_count", &v)) info->agprs = (int)v;
    if (find_uint(image, ".sgpr_count", &v)) info->sgprs = (int)v;
    if (find_uint(image, ".group_segment_fixed_size", &v)) info->lds_bytes = (int)v;
    if (find_uint(image, ".private_segment_fixed_size", &v)) info->scratch_bytes = (int)v;
}

// The kernel source with comments removed, runs of blanks collapsed and blank lines dropped:
// what the cache key is computed from, so that rewording a comment does not invalidate every
// cached variant.  Line breaks are kept (they end preprocessor directives).
std::string normalize(const char *p, const char *end) {
    std::string out;
    out.reserve((size_t)(end - p));
    int gap = 0; // 0 = none, 1 = blanks, 2 = at least one line break
    while (p < end) {
        if (p + 1 < end && p[0] == '/' && p[1] == '/') {
            while (p < end && *p != '\n') ++p;
        } else if (p + 1 < end && p[0] == '/' && p[1] == '*') {
            p += 2;
            while (p + 1 < end && !(p[0] == '*' && p[1] == '/')) ++p;
            p = (p + 1 < end) ? p + 2 : end;
            if (gap < 1) gap = 1;
        } else if (*p == '\n') {
            gap = 2;
            ++p;
        } else if (*p == ' ' || *p == '\t' || *p == '\r') {
            if (gap < 1) gap = 1;
            ++p;
        } else {
            if (gap && !out.empty()) out.push_back(gap == 2 ? '\n' : ' ');
            gap = 0;
            out.push_back(*p++);
        }
    }
    return out;
}

// The two built-in families are normalised once; a caller-supplied source each time it is used.
std::string normalized_source(const KernelSource &src) {
    static const std::string gemm = normalize(sgemm_kernel_source_begin, sgemm_kernel_source_end);
    static const std::string conv = normalize(conv_kernel_source_begin, conv_kernel_source_end);
    if (src.begin == sgemm_kernel_source_begin) return gemm;
    if (src.begin == conv_kernel_source_begin) return conv;
    return normalize(src.begin, src.end) + "\n" + src.entry;
}

const KernelSource &gemm_source() {
    static const KernelSource s{sgemm_kernel_source_begin, sgemm_kernel_source_end, "sgemm_variant.hip",
                                "sgemm_variant"};
    return s;
}

const KernelSource &conv_source() {
    static const KernelSource s{conv_kernel_source_begin, conv_kernel_source_end, "conv2d_variant.hip",
                                "conv2d_variant"};
    return s;
}

// File of a variant's code object in the cache directory: a hash of the kernel source (without
// comments), the macros, the compiler flags, any experiment defines and the compiler's identity.
std::string code_object_path(const VariantKey &key) { return code_object_path(gemm_source(), key.macros()); }

std::string code_object_path(const KernelSource &source, const std::string &macros) {
    const std::string src = normalized_source(source);
    uint64_t h = fnv1a(src.data(), src.size());
    h = fnv1a(macros.data(), macros.size(), h);
    for (const char *f : kCompilerFlags) h = fnv1a(f, std::strlen(f), h);
    // extra -D options for kernel experiments (space separated); part of the cache key
    const char *extra_env = std::getenv("SGEMM_TUNED_EXTRA_DEFINES");
    const std::string extra = extra_env ? extra_env : "";
    h = fnv1a(extra.data(), extra.size(), h);
    h = compiler_identity(h);
    char name[40];
    std::snprintf(name, sizeof name, "/%016llx.hsaco", (unsigned long long)h);
    return cache_dir() + name;
}

int get_code_object(const VariantKey &key, CodeObject *out, std::string *log) {
    return get_code_object(gemm_source(), key.macros(), out, log);
}

int get_code_object(const KernelSource &source, const std::string &macros, CodeObject *out,
                    std::string *log) {
    const char *extra_env = std::getenv("SGEMM_TUNED_EXTRA_DEFINES");
    const std::string extra = extra_env ? extra_env : "";
    const std::string path = code_object_path(source, macros);
    const std::string dir = cache_dir();

    out->info = sgemm_kernel_info{};
    if (read_file(path, &out->image)) {
        read_code_object_info(out->image, &out->info);
        out->info.from_cache = 1;
        return SGEMM_OK;
    }

    const auto t0 = std::chrono::steady_clock::now();
    // split the macro string into separate options
    std::vector<std::string> opts;
    for (const char *f : kCompilerFlags) opts.emplace_back(f);
    {
        size_t pos = 0;
        while (pos < macros.size()) {
            size_t sp = macros.find(' ', pos);
            if (sp == std::string::npos) sp = macros.size();
            if (sp > pos) opts.emplace_back(macros.substr(pos, sp - pos));
            pos = sp + 1;
        }
    }
    {
        size_t pos = 0;
        while (pos < extra.size()) {
            size_t sp = extra.find(' ', pos);
            if (sp == std::string::npos) sp = extra.size();
            if (sp > pos) opts.emplace_back(extra.substr(pos, sp - pos));
            pos = sp + 1;
        }
    }
    std::vector<const char *> argv;
    for (auto &o : opts) argv.push_back(o.c_str());

    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, source.begin, source.file_name, 0, nullptr,
                            nullptr) != HIPRTC_SUCCESS) {
        if (log) *log = "hiprtcCreateProgram failed";
        return SGEMM_E_COMPILE;
    }
    const hiprtcResult rc = hiprtcCompileProgram(prog, (int)argv.size(), argv.data());
    if (rc != HIPRTC_SUCCESS) {
        if (log) {
            size_t n = 0;
            hiprtcGetProgramLogSize(prog, &n);
            log->assign(n, '\0');
            if (n) hiprtcGetProgramLog(prog, &(*log)[0]);
            *log = std::string(hiprtcGetErrorString(rc)) + " [" + macros + "]\n" + *log;
        }
        hiprtcDestroyProgram(&prog);
        return SGEMM_E_COMPILE;
    }
    size_t size = 0;
    hiprtcGetCodeSize(prog, &size);
    out->image.resize(size);
    hiprtcGetCode(prog, out->image.data());
    hiprtcDestroyProgram(&prog);
    const auto t1 = std::chrono::steady_clock::now();

    read_code_object_info(out->image, &out->info);
    out->info.from_cache = 0;
    out->info.compile_ms = std::chrono::duration<float, std::milli>(t1 - t0).count();
    mkdir(dir.c_str(), 0777);
    write_file_atomic(path, out->image);
    return SGEMM_OK;
}

LoadedKernel::~LoadedKernel() {
    if (module) (void)hipModuleUnload(module);
}

int load_kernel(const VariantKey &key, std::shared_ptr<LoadedKernel> *out, std::string *log) {
    return load_kernel(gemm_source(), key.macros(), threads_of(key.cfg), out, log);
}

int load_kernel(const KernelSource &source, const std::string &macros, int threads,
                std::shared_ptr<LoadedKernel> *out, std::string *log) {
    CodeObject co;
    const int rc = get_code_object(source, macros, &co, log);
    if (rc != SGEMM_OK) return rc;
    auto k = std::make_shared<LoadedKernel>();
    k->info = co.info;
    k->threads = threads;
    hipError_t e = hipModuleLoadData(&k->module, co.image.data());
    if (e != hipSuccess) {
        if (log) *log = std::string("hipModuleLoadData: ") + hipGetErrorString(e) + " [" + macros + "]";
        k->module = nullptr;
        return SGEMM_E_LAUNCH;
    }
    e = hipModuleGetFunction(&k->fn, k->module, source.entry);
    if (e != hipSuccess) {
        if (log) *log = std::string("hipModuleGetFunction: ") + hipGetErrorString(e);
        return SGEMM_E_LAUNCH;
    }
    *out = std::move(k);
    return SGEMM_OK;
}

} // namespace sgemm
