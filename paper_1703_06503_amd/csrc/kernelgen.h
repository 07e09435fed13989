// Kernel generator: turns one configuration into a gfx950 code object by compiling the
// embedded kernel source with the configuration as -D macros (hipRTC), keeps code objects in
// an on-disk cache, and loads them as HIP modules.  The paper recompiles its kernel once per
// configuration in the same way (section "CLTune: an auto-tuner for OpenCL kernels") and
// notes that recompilation can dominate tuning time ("Search strategies ..."): hence the cache.
#pragma once
#include <hip/hip_runtime_api.h>

#include <memory>
#include <string>
#include <vector>

#include "../../include/sgemm_tuned.h"

namespace sgemm {

// The variant actually built for a call: configuration + storage layout + guarded or not.
struct VariantKey {
    sgemm_config cfg;
    int layout;
    int edge;
    int splitk = 0; // 1 = the build that split-K launches use (cfg.sk itself is not compiled in)
    int cpf = 0;    // 1 = the build for beta != 0 that requests the old C before the first slab
    std::string macros() const; // "-DMWG=.. -DNWG=.. ..." in a fixed order
};

// A kernel family's source text as it travels inside the library, and its entry point.
struct KernelSource {
    const char *begin, *end;
    const char *file_name; // name shown in compiler messages
    const char *entry;
};
const KernelSource &gemm_source(); // sgemm_kernel.hip.inc
const KernelSource &conv_source(); // conv_kernel.hip.inc

struct CodeObject {
    std::vector<char> image;
    sgemm_kernel_info info{};
};

// Compile or fetch from the disk cache.  Needs no GPU.  On failure returns SGEMM_E_COMPILE
// and, if log is non-null, the compiler's message.
int get_code_object(const VariantKey &key, CodeObject *out, std::string *log);

// Where the variant's code object is (or will be) kept in the cache directory.
std::string code_object_path(const VariantKey &key);

// The same three steps for any kernel family: `macros` is its "-DNAME=value ..." string.
int get_code_object(const KernelSource &source, const std::string &macros, CodeObject *out,
                    std::string *log);
std::string code_object_path(const KernelSource &source, const std::string &macros);

void set_cache_dir(const std::string &path);
std::string cache_dir();

// A loaded variant; unloads its module when destroyed.
struct LoadedKernel {
    hipModule_t module = nullptr;
    hipFunction_t fn = nullptr;
    sgemm_kernel_info info{};
    int threads = 0;
    ~LoadedKernel();
};

int load_kernel(const VariantKey &key, std::shared_ptr<LoadedKernel> *out, std::string *log);
int load_kernel(const KernelSource &source, const std::string &macros, int threads,
                std::shared_ptr<LoadedKernel> *out, std::string *log);

// Reads vgpr/agpr/sgpr counts and LDS/scratch sizes from a code object's metadata note.
void read_code_object_info(const std::vector<char> &image, sgemm_kernel_info *info);

} // namespace sgemm
