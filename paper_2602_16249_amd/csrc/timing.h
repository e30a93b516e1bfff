// Optional per-kernel timing with HIP events on the launch stream.  Disabled by
// default (then a timed launch is just the launch).  Used by the benchmark to
// report the duration of individual kernels inside one API call.
#pragma once

#include <hip/hip_runtime.h>

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

// Launch a kernel, bracketed by timing events when timing is enabled.
#define AFFMAE_LAUNCH(name, stream, ...)            \
  do {                                              \
    ::affmae::TimedScope affmae_ts_(name, stream);  \
    hipLaunchKernelGGL(__VA_ARGS__);                \
  } while (0)
