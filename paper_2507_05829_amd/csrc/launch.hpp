// One place where kernels are launched, so that a launch can carry the events that time it.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace lop {

// Launches `kernel`; with `ev` the next free (start, stop) pair is attached to the dispatch
// itself, so their difference is the kernel's own duration as a profiler reports it (an event
// recorded before and after a launch also spans the gaps between dispatches).
template <typename... KArgs, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s,
                                KernelEvents* ev, Args... args) {
  if (ev && ev->n < KernelEvents::kMax) {
    const int i = ev->n++;
    hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ev->start[i], ev->stop[i], 0,
                          static_cast<KArgs>(args)...);
  } else {
    hipLaunchKernelGGL(kernel, grid, block, 0, s, static_cast<KArgs>(args)...);
  }
  return hipGetLastError();
}

}  // namespace lop
