// Pieces of the tuning harness that every kernel family of the library uses: the calling
// thread's error text, the library's stream, device buffers and events that clean up after
// themselves, search parameters from the caller's options, and the timing of one configuration
// (paper: "CLTune: an auto-tuner for OpenCL kernels" -- each configuration is run, verified and
// timed in the same way whatever the kernel).
#pragma once
#include <hip/hip_runtime_api.h>

#include <functional>
#include <string>
#include <vector>

#include "../../include/sgemm_tuned.h"
#include "strategy.h"

namespace sgemm {
namespace detail {

void set_error(const std::string &what);
hipStream_t library_stream(); // the stream given to sgemm_set_stream()

struct DeviceBuffer {
    void *p = nullptr;
    ~DeviceBuffer() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 4); }
    float *f() const { return static_cast<float *>(p); }
};

struct Event {
    hipEvent_t e = nullptr;
    Event() { (void)hipEventCreate(&e); }
    ~Event() { if (e) (void)hipEventDestroy(e); }
};

double median(std::vector<double> v);
StrategyParams params_from(const tune_opts *o);

// How one configuration is timed once its first, verified launch has taken first_ms: launches
// without timing until the clock has settled (at least warmup - 1 of them and about warmup_ms
// of GPU time), then `reps` samples of enough launches each to last 0.2 ms, of which the median
// is kept.  A configuration slower than cut x best_ms (cut > 0 and best_ms > 0) is dropped
// early: before the warm-up when even its cold first launch allows it, else after the first
// sample; its time is then that one measurement and *was_cut is set.
// Returns milliseconds per launch, or a negative value after a device failure.
struct TimingRules {
    int warmup = 2;
    int reps = 7;
    double warmup_ms = 25.0;
    double cut = 3.0;
};
TimingRules timing_rules_from(const tune_opts *o);
double time_configuration(hipStream_t s, const std::function<void()> &launch, float first_ms,
                          const TimingRules &rules, double best_ms, Event &ev0, Event &ev1,
                          int *samples, bool *was_cut);

// The part of an evaluation that is the same for every kernel family, once the variant is loaded:
// give the kernel fresh arguments, run it once between two events, compare its outputs with the
// reference's, and time it by the rules above.
//   fresh_arguments  restores whatever the kernel overwrites (may be empty)
//   launch           one launch on s; false when HIP refused it
//   outputs_differ   enqueues the comparison(s), waits for the stream and returns 1 when an
//                    output is outside its bound, 0 when all match, -1 when the device failed;
//                    empty = no verification (the stream is still waited for)
// status is "ok", "ok-cut" (timed, but dropped early as hopeless), "launch", "verify" or "fault";
// after "fault" the device is not to be used further (device_failed).  ms < 0 unless timed.
struct Measured {
    double ms = -1.0;
    const char *status = "ok";
    int samples = 0;
    bool device_failed = false;
};
Measured run_verify_time(hipStream_t s, const std::function<void()> &fresh_arguments,
                         const std::function<bool()> &launch, const std::function<int()> &outputs_differ,
                         const TimingRules &rules, double best_ms, Event &ev0, Event &ev1);

} // namespace detail
} // namespace sgemm
