// Host-side launch helper shared by every translation unit of the library.
//
// nf_launch() enqueues one kernel.  When the calling thread has armed a pair of timing events with
// netfuse_time_next_launch(), that one launch goes through hipExtLaunchKernelGGL, which binds the events to
// the kernel's own begin and end timestamps on the device (what a kernel trace reports), and the request
// is cleared; every other launch is a plain hipLaunchKernelGGL.
//
// dev_getenv(): developer switches for sweeps and A/B runs.  They exist only in builds that define
// NETFUSE_DEV_SWITCHES; the library as shipped reads no environment variable.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdlib.h>

namespace nf {

struct LaunchTiming {
  hipEvent_t start, stop;
};
// the calling thread's pending request (both null = none); defined in netfuse_api.hip
LaunchTiming& launch_timing();

template <class Kernel, class... Args>
inline void nf_launch(Kernel kern, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s, Args... args) {
  LaunchTiming& t = launch_timing();
  if (t.start != nullptr || t.stop != nullptr) {
    hipExtLaunchKernelGGL(kern, grid, block, lds_bytes, s, t.start, t.stop, 0, args...);
    t.start = nullptr;
    t.stop = nullptr;
  } else {
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, s, args...);
  }
}

#ifdef NETFUSE_DEV_SWITCHES
inline const char* dev_getenv(const char* name) { return getenv(name); }
#else
inline const char* dev_getenv(const char*) { return nullptr; }
#endif

}  // namespace nf
