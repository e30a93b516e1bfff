// Kernel launch macro.  The product library (libaffmae.so) is built without AFFMAE_TIMING: a launch is just the
// launch and the library holds no state between calls.  The instrumented build (libaffmae_timed.so, compiled with
// -DAFFMAE_TIMING, loaded only by the benchmark) brackets every launch with two HIP events on the launch stream and
// keeps per-kernel totals in a registry (timing.hip, declared in include/affmae_timing.h).
#pragma once

#include <hip/hip_runtime.h>

#ifdef AFFMAE_TIMING
namespace affmae {

bool timing_enabled();
void timing_begin(const char* name, hipStream_t stream);
void timing_end(hipStream_t stream);

struct TimedScope {
  hipStream_t s;
  bool on;
  TimedScope(const char* name, hipStream_t stream) : s(stream), on(timing_enabled()) {
    if (on) timing_begin(name, s);
  }
  ~TimedScope() {
    if (on) timing_end(s);
  }
};

}  // namespace affmae

#define AFFMAE_LAUNCH(name, stream, ...)            \
  do {                                              \
    ::affmae::TimedScope affmae_ts_(name, stream);  \
    hipLaunchKernelGGL(__VA_ARGS__);                \
  } while (0)
#else
#define AFFMAE_LAUNCH(name, stream, ...) hipLaunchKernelGGL(__VA_ARGS__)
#endif
