// One place through which the main-pass kernels are launched, so that a caller can have a
// launch timed by the runtime itself: when a pair of events is armed, the launch goes through
// hipExtLaunchKernelGGL, which stamps them with the kernel's own begin and end (no stream
// markers around it, so neither their cost nor the gap between launches is in the interval).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace bd {

extern hipEvent_t g_launch_events[2];  // armed by bcast_dual_set_launch_events, cleared by the launch that uses them

template <class K, class... A>
inline void launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, const A &...args) {
  (void)hipGetLastError();  // the callers read the error state after the launch: an earlier, unrelated call's must not be in it
  if (g_launch_events[0] != nullptr) {
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, g_launch_events[0], g_launch_events[1], 0u, args...);
    g_launch_events[0] = g_launch_events[1] = nullptr;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
  }
}

}  // namespace bd
