// What this GPU sustains on the two resources the kernels are priced against: a plain copy
// through HBM and a loop of nothing but MFMAs. Measurement aid: the published peaks are the
// roofline's denominators, these figures say how much of them any kernel can reach here.
#include <hip/hip_runtime.h>

#include "lop.h"
#include "launch.hpp"
#include "plan_state.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyBlocks = 256 * 8;   // eight workgroups per compute unit
constexpr int kMfmaChains = 4;         // independent accumulators per wavefront
constexpr int kMfmaIters = 4096;

// n 16-byte vectors from src to dst, grid-stride, consecutive lanes on consecutive vectors
// (four strided loads in flight per thread were slower: 4.4 against 4.9 TB/s)
__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                   size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Operand bits that differ per lane and look like data (all-zero operands let the chip clock
// higher than any real tile does).
__device__ __forceinline__ unsigned mix(unsigned v) {
  v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
  return v;
}

// kMfmaIters rounds of kMfmaChains independent 32x32x16 bf16 MFMAs per wavefront; the sums go
// to `sink` so the loop is not removed.
__global__ __launch_bounds__(256) void mfma_bf16_kernel(float* __restrict__ sink) {
  const unsigned seed = blockIdx.x * 256 + threadIdx.x;
  // bf16 values in (-2, 2): sign and mantissa from the hash, exponent fixed
  auto operand = [&](unsigned salt) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (mix(seed * 4 + i + salt) & 0x807f807fu) | 0x3f803f80u;
    return __builtin_bit_cast(bf16x8, v);
  };
  const bf16x8 a = operand(1), b = operand(2);
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < kMfmaIters; ++it)
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// the same with 32x32x2 fp32 MFMAs
__global__ __launch_bounds__(256) void mfma_f32_kernel(float* __restrict__ sink) {
  const unsigned seed = blockIdx.x * 256 + threadIdx.x;
  const float a = __builtin_bit_cast(float, (mix(seed + 11) & 0x807fffffu) | 0x3f800000u);
  const float b = __builtin_bit_cast(float, (mix(seed + 29) & 0x807fffffu) | 0x3f800000u);
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < kMfmaIters; ++it)
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

struct Buffers {
  void *a = nullptr, *b = nullptr;
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ~Buffers() {
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    if (sink) (void)hipFree(sink);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

// Returns at once (the argument only gives the launch something to pass).
__global__ void empty_kernel(float* sink) { (void)sink; }

}  // namespace

extern "C" int lop_measure_ceilings(lop_ceilings_t* out) {
  if (!out) return LOP_ERR_INVALID_ARG;
  constexpr size_t kBytes = (size_t)1 << 30;  // per buffer: far beyond the 256 MB last-level cache
  constexpr int kWaveGrid = 256 * 2;          // workgroups of four wavefronts: two wavefronts per SIMD
  Buffers B;
  LOP_HIP(hipMalloc(&B.a, kBytes));
  LOP_HIP(hipMalloc(&B.b, kBytes));
  LOP_HIP(hipMalloc((void**)&B.sink, (size_t)kWaveGrid * 256 * sizeof(float)));
  LOP_HIP(hipMemset(B.a, 1, kBytes));
  LOP_HIP(hipEventCreate(&B.e0));
  LOP_HIP(hipEventCreate(&B.e1));
  float ms = 0.f;
  auto timed = [&](auto&& launch, int reps, float* best) -> int {
    *best = 1e30f;
    launch();  // warm-up
    for (int r = 0; r < reps; ++r) {
      LOP_HIP(hipEventRecord(B.e0, nullptr));
      launch();
      LOP_HIP(hipEventRecord(B.e1, nullptr));
      LOP_HIP(hipEventSynchronize(B.e1));
      LOP_HIP(hipEventElapsedTime(&ms, B.e0, B.e1));
      *best = ms < *best ? ms : *best;
    }
    return hipGetLastError() == hipSuccess ? LOP_OK : LOP_ERR_HIP;
  };
  float t = 0.f;
  int rc = timed([&] { hipLaunchKernelGGL(copy_kernel, dim3(kCopyBlocks), dim3(256), 0, nullptr, (u32x4*)B.b,
                                          (const u32x4*)B.a, kBytes / 16); }, 5, &t);
  if (rc != LOP_OK) return rc;
  out->hbm_copy_gbs = 2.0 * kBytes / (t * 1e-3) / 1e9;  // bytes read + bytes written
  const double waves = (double)kWaveGrid * 4;
  rc = timed([&] { hipLaunchKernelGGL(mfma_bf16_kernel, dim3(kWaveGrid), dim3(256), 0, nullptr, B.sink); }, 5, &t);
  if (rc != LOP_OK) return rc;
  out->mfma_bf16_tflops = waves * kMfmaIters * kMfmaChains * (2.0 * 32 * 32 * 16) / (t * 1e-3) / 1e12;
  rc = timed([&] { hipLaunchKernelGGL(mfma_f32_kernel, dim3(kWaveGrid), dim3(256), 0, nullptr, B.sink); }, 5, &t);
  if (rc != LOP_OK) return rc;
  out->mfma_f32_tflops = waves * kMfmaIters * kMfmaChains * (2.0 * 32 * 32 * 2) / (t * 1e-3) / 1e12;
  // what a launch costs before it does anything: a kernel of 128 workgroups that returns at
  // once, timed by events attached to the dispatch like every per-launch figure of the library
  {
    lop::KernelEvents ev;
    LOP_HIP(hipEventCreate(&ev.start[0]));
    LOP_HIP(hipEventCreate(&ev.stop[0]));
    double sum = 0.0;
    constexpr int kReps = 20;
    for (int r = 0; r < kReps + 1; ++r) {
      ev.n = 0;
      LOP_HIP(lop::launch_kernel(empty_kernel, dim3(128), dim3(256), nullptr, &ev, B.sink));
      LOP_HIP(hipEventSynchronize(ev.stop[0]));
      LOP_HIP(hipEventElapsedTime(&ms, ev.start[0], ev.stop[0]));
      if (r > 0) sum += ms;   // (the first one warms up)
    }
    out->launch_floor_us = sum / kReps * 1e3;
    (void)hipEventDestroy(ev.start[0]);
    (void)hipEventDestroy(ev.stop[0]);
  }
  // ... and the same kernel as 200 dependent nodes of a graph replayed on one stream (how the
  // chains run in steady state): wall time per node
  {
    constexpr int kNodes = 200, kReplays = 5;
    hipStream_t st = nullptr;
    hipGraph_t g = nullptr;
    hipGraphExec_t ex = nullptr;
    LOP_HIP(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    LOP_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    for (int i = 0; i < kNodes; ++i) hipLaunchKernelGGL(empty_kernel, dim3(128), dim3(256), 0, st, B.sink);
    hipError_t e = hipStreamEndCapture(st, &g);
    if (e == hipSuccess) e = hipGraphInstantiate(&ex, g, nullptr, nullptr, 0);
    if (g) (void)hipGraphDestroy(g);
    if (e == hipSuccess) e = hipGraphLaunch(ex, st);   // warm-up
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipEventRecord(B.e0, st);
    for (int r = 0; r < kReplays && e == hipSuccess; ++r) e = hipGraphLaunch(ex, st);
    if (e == hipSuccess) e = hipEventRecord(B.e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(B.e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, B.e0, B.e1);
    if (ex) (void)hipGraphExecDestroy(ex);
    (void)hipStreamDestroy(st);
    LOP_HIP(e);
    out->graph_node_floor_us = ms * 1e3 / (kNodes * kReplays);
  }
  LOP_HIP(hipDeviceSynchronize());
  return LOP_OK;
}
