// One place through which the main-pass kernels are launched, so that a caller can have a
// launch timed by the runtime itself: with a pair of events in `L` the launch goes through
// hipExtLaunchKernelGGL, which stamps them with the kernel's own begin and end (no stream
// markers around it, so neither their cost nor the gap between launches is in the interval).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "launch_types.h"

namespace bd {

template <class K, class... A>
inline void launch(K kernel, dim3 grid, dim3 block, size_t lds, const Launch &L, const A &...args) {
  (void)hipGetLastError();  // the callers read the error state after the launch: an earlier, unrelated call's must not be in it
  if (L.start != nullptr)
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, L.stream, L.start, L.stop, 0u, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, L.stream, args...);
}

}  // namespace bd
