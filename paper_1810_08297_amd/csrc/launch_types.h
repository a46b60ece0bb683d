// Where a kernel is enqueued: the caller's stream and, optionally, a pair of the caller's events
// that the launch stamps with the kernel's own begin and end.
#pragma once
#include <hip/hip_runtime_api.h>

namespace bd {

struct Launch {
  hipStream_t stream;
  hipEvent_t start, stop;  // both null: an ordinary launch
};

}  // namespace bd
