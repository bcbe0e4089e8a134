// Activation as a clamp: none = [-inf, +inf], ReLU = [0, +inf], ReLU6 = [0, 6]. The bounds
// are chosen once per kernel from the runtime activation code and applied with one
// median-of-three instruction per value, instead of a branch per value.
#pragma once
#include <hip/hip_runtime.h>

#include "lop.h"

namespace lop {

struct Clamp {
  float lo, hi;
};

__host__ __device__ __forceinline__ Clamp make_clamp(int act) {
  Clamp c;
  c.lo = act == LOP_ACT_NONE ? -INFINITY : 0.f;
  c.hi = act == LOP_ACT_RELU6 ? 6.f : INFINITY;
  return c;
}

__device__ __forceinline__ float clamp_act(float v, const Clamp& c) {
  return __builtin_amdgcn_fmed3f(v, c.lo, c.hi);
}

}  // namespace lop
