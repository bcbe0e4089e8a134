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

// Several launches of one operator - the bands of a chain at one layer - as one grid (the
// operation batching of Sec. IV-D: the local operations a device holds of one operator go
// into one kernel call). Band b owns the blocks first[b] .. first[b + 1] of the grid's x
// dimension and has its own parameters; y and z extents are the same for every band.
constexpr int kMaxBatch = 16;
template <typename P>
struct Batch {
  int n;
  int first[kMaxBatch + 1];
  P p[kMaxBatch];
};
template <typename P>
__device__ __forceinline__ int batch_find(const Batch<P>& t, int bx) {
  int b = 0;
  while (b + 1 < t.n && bx >= t.first[b + 1]) ++b;
  return b;
}

// One band: the kernel itself; several bands of the layer: its _bands form on a grid whose x
// extent is the sum of the bands' (gx: blocks of x per band).
template <typename P>
inline hipError_t launch_group(void (*single)(const P), void (*bands)(const Batch<P>), const P* ps, int n,
                               const unsigned* gx, unsigned gy, unsigned gz, dim3 block, hipStream_t s,
                               KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch || gy > 65535 || gz > 65535) return hipErrorInvalidValue;
  if (n == 1) return launch_kernel(single, dim3(gx[0], gy, gz), block, s, ev, ps[0]);
  Batch<P> t;
  t.n = n;
  unsigned long at = 0;
  for (int b = 0; b < kMaxBatch; ++b) {
    t.first[b] = (int)at;
    t.p[b] = ps[b < n ? b : n - 1];
    if (b < n) at += gx[b];
  }
  t.first[kMaxBatch] = (int)at;
  if (at == 0 || at > 0x7fffffffUL) return hipErrorInvalidValue;
  return launch_kernel(bands, dim3((unsigned)at, gy, gz), block, s, ev, t);
}

}  // namespace lop
