// 1x1 stride-1 convolution = the row-wise local operator (Intra-DP Sec. IV-A, Eq. 1): every
// output pixel is its own input row times the whole weight matrix, so a row band needs no
// halo at all. With few channels this is a bandwidth-bound stream, not a GEMM to tile: each
// wavefront keeps the entire weight matrix in registers as MFMA operand fragments, takes a
// few groups of 32 pixels, loads their channels straight from global memory in the operand
// layout (no LDS staging), multiplies, and turns each accumulator tile through a small
// wave-private LDS region so that every store and residual load is a contiguous 16-byte
// piece per lane. All loads of a wavefront are issued before its first store: on this
// architecture loads and stores share one in-order counter, so a load waited for after a
// store would also wait for the store to be acknowledged.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>

#include "act.hpp"
#include "kernels.hpp"
#include "launch.hpp"
#include "lop.h"

namespace lop {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct PwParams {
  const __bf16* x;
  __bf16* y;
  const __bf16* res;
  const __bf16* w;  // [c_out_pad][k_pad]
  const float* bias;
  int x_row0, x_rows, W, C_in;
  int y_row0, y_rows, C_out;
  int r_row0, r_rows;
  int act, out_lo, R, N;
  int M;  // N * R * W
  int k_pad;
  int groups;  // ceil(M / 32)
  int iters;   // groups per wavefront
};

// The staging rows are private to a wavefront and the LDS executes one wavefront's
// instructions in issue order, so a write followed by a read of another lane's data needs
// no barrier: only the compiler has to be kept from reordering the two.
__device__ __forceinline__ void lds_wave_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// NT: 32-channel tiles of the output (C_out = 32 * NT); KS: 16-element steps of the
// reduction (C_in = 16 * KS); RES: a residual is added (its loads are the only loads
// issued after the first store; without it the store stream is never waited for).
template <int NT, int KS, bool RES>
__global__ __launch_bounds__(256) void pointwise_kernel(const PwParams p) {
  constexpr int CH = NT >= 2 ? 2 : 1;   // tiles turned through LDS at a time
  constexpr int CP = CH * 32 + 4;       // fp32 pitch of the staged rows
  __shared__ __attribute__((aligned(16))) float stage[4][32 * CP];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int px = lane & 31, kg = lane >> 5;
  float* const st = stage[wave];
  const Clamp clamp = make_clamp(p.act);

  // the whole weight matrix as A-operand fragments: tile t, step s -> channels t*32+px,
  // reduction elements s*16 + kg*8 .. +8
  uint4 wf[NT][KS];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < KS; ++s)
      wf[t][s] = *(const uint4*)(p.w + (size_t)(t * 32 + px) * p.k_pad + s * 16 + kg * 8);

  constexpr int GPW = KS >= 8 ? 1 : 2;  // pixel groups per wavefront
  const int wid = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(wave);

  // A band of a 1x1 stride-1 layer is one contiguous run of pixels per image in the input,
  // output and residual slabs alike, so a pixel's address is linear in its index m once
  // the image n = m / (R*W) is known: off(m) = (n*img + first + (m - n*R*W)) * channels.
  const int RW = p.R * p.W;
  const long x_img = (long)p.x_rows * p.W, x_first = (long)(p.out_lo - p.x_row0) * p.W;
  const long y_img = (long)p.y_rows * p.W, y_first = (long)(p.out_lo - p.y_row0) * p.W;
  const long r_img = (long)p.r_rows * p.W, r_first = (long)(p.out_lo - p.r_row0) * p.W;

  // image of pixel m of group g: one division per group (wave-uniform); a group spans at
  // most two images when an image's band holds at least 32 pixels
  auto image_of = [&](int g, int m) -> int {
    if (RW < 32) return m / RW;
    const int n0 = (g * 32) / RW;
    return n0 + (m >= (n0 + 1) * RW ? 1 : 0);
  };
  auto load_group = [&](int g, uint4 (&a)[KS]) {
    const int m = g * 32 + px;
    if (g < p.groups && m < p.M) {
      const int n = image_of(g, m);
      const __bf16* src = p.x + (size_t)(n * x_img + x_first + (m - n * RW)) * p.C_in + kg * 8;
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = *(const uint4*)(src + s * 16);
    } else {
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = make_uint4(0, 0, 0, 0);
    }
  };

  // Epilogue ownership (fixed for the whole kernel): in a turn of `tiles` 32-channel tiles
  // a pixel has VPP = 4*tiles 16-byte pieces; lane owns piece v = lane % VPP of pixels
  // q = lane / VPP + j * (64 / VPP). Its bias values never change.
  constexpr int TURNS = (NT + CH - 1) / CH;
  float bias[TURNS][8];
#pragma unroll
  for (int tu = 0; tu < TURNS; ++tu) {
    const int tiles = (NT - tu * CH) < CH ? (NT - tu * CH) : CH;
    const int co = tu * CH * 32 + (lane % (tiles * 4)) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) bias[tu][i] = p.bias ? p.bias[co + i] : 0.f;
  }

  uint4 grp[GPW][KS];
#pragma unroll
  for (int i = 0; i < GPW; ++i) load_group(wid * GPW + i, grp[i]);
  // Every load above is waited for here, before the first store is issued: loads and
  // stores share one in-order counter, so a load consumed inside the loop below would
  // make every iteration wait for the previous iteration's stores as well.
#pragma unroll
  for (int i = 0; i < GPW; ++i)
#pragma unroll
    for (int s = 0; s < KS; ++s)
      asm volatile("" ::"v"(grp[i][s].x), "v"(grp[i][s].y), "v"(grp[i][s].z), "v"(grp[i][s].w));
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < KS; ++s)
      asm volatile("" ::"v"(wf[t][s].x), "v"(wf[t][s].y), "v"(wf[t][s].z), "v"(wf[t][s].w));
#pragma unroll
  for (int tu = 0; tu < TURNS; ++tu)
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(bias[tu][i]));
  for (int it = 0; it < GPW; ++it) {  // not unrolled: the body is long
    const int g = wid * GPW + it;
    uint4 cur[KS];  // grp[it], selected with static register indices
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      cur[s] = grp[0][s];
#pragma unroll
      for (int i = 1; i < GPW; ++i)
        if (it == i) cur[s] = grp[i][s];
    }

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[t][s]),
                                                         __builtin_bit_cast(bf16x8, cur[s]),
                                                         acc[t], 0, 0, 0);

    // ---- epilogue, CH tiles (32*CH channels) at a time through this wave's LDS rows.
    // Accumulator layout: pixel px, channels g8*8 + kg*4 + {0..3} of the tile, g8 = 0..3.
#pragma unroll
    for (int tu = 0; tu < TURNS; ++tu) {
      const int c0 = tu * CH;
      const int tiles = (NT - c0) < CH ? (NT - c0) : CH;
      const int VPP = tiles * 4, QSTEP = 64 / VPP;
      lds_wave_order();  // the previous turn's reads are issued before these writes
#pragma unroll
      for (int t = 0; t < CH; ++t) {
        if (c0 + t < NT) {
#pragma unroll
          for (int g8 = 0; g8 < 4; ++g8)
            *(float4*)(st + px * CP + t * 32 + g8 * 8 + kg * 4) =
                make_float4(acc[c0 + t][g8 * 4], acc[c0 + t][g8 * 4 + 1], acc[c0 + t][g8 * 4 + 2],
                            acc[c0 + t][g8 * 4 + 3]);
        }
      }
      lds_wave_order();
      const int v = lane % VPP, q0 = lane / VPP;
      // Addresses: one wave-uniform base per group plus a 32-bit per-lane offset. Pixel
      // m0 + q lies `wraps` images after image n0; each image adds (img - R*W) pixels of
      // rows outside the band to the linear offset.
      const int m0 = g * 32;
      const int n0 = m0 / RW, rem0 = m0 - n0 * RW;
      __bf16* const ybase = p.y + ((size_t)n0 * y_img + y_first + rem0) * p.C_out + c0 * 32 + v * 8;
      const __bf16* const rbase =
          RES ? p.res + ((size_t)n0 * r_img + r_first + rem0) * p.C_out + c0 * 32 + v * 8 : nullptr;
      constexpr int JN = 32 / (64 / ((CH < 2 ? 1 : 2) * 4));  // upper bound of slots per lane
      uint4 rres[JN];
      int wraps_j[JN];
#pragma unroll
      for (int j = 0; j < 32 / QSTEP; ++j) {
        const int q = q0 + j * QSTEP;
        wraps_j[j] = RW >= 32 ? (rem0 + q >= RW ? 1 : 0) : (rem0 + q) / RW;
        rres[j] = make_uint4(0, 0, 0, 0);
        if constexpr (RES) {
          if (g < p.groups && m0 + q < p.M)
            rres[j] = *(const uint4*)(rbase + (q + wraps_j[j] * (int)(r_img - RW)) * p.C_out);
        }
      }
      if constexpr (RES) {  // one wait for the turn's residual vectors
#pragma unroll
        for (int j = 0; j < 32 / QSTEP; ++j)
          asm volatile("" ::"v"(rres[j].x), "v"(rres[j].y), "v"(rres[j].z), "v"(rres[j].w));
      }
#pragma unroll
      for (int j = 0; j < 32 / QSTEP; ++j) {
        const int q = q0 + j * QSTEP;
        if (g >= p.groups || m0 + q >= p.M) continue;
        const float4 lo = *(const float4*)(st + q * CP + v * 8);
        const float4 hi = *(const float4*)(st + q * CP + v * 8 + 4);
        float o[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] += bias[tu][i];
        if constexpr (RES) {
          const unsigned u[4] = {rres[j].x, rres[j].y, rres[j].z, rres[j].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            o[2 * i] += __uint_as_float(u[i] << 16);
            o[2 * i + 1] += __uint_as_float(u[i] & 0xffff0000u);
          }
        }
        alignas(16) __bf16 ob[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) ob[i] = (__bf16)clamp_act(o[i], clamp);
        *(uint4*)(ybase + (q + wraps_j[j] * (int)(y_img - RW)) * p.C_out) = *(const uint4*)ob;
      }
    }
  }
}

template <int NT, int KS>
hipError_t launch_pw(PwParams& p, hipStream_t s, KernelEvents* ev) {
  constexpr int GPW = KS >= 8 ? 1 : 2;  // must match the kernel
  const int waves = (p.groups + GPW - 1) / GPW;
  const int grid = std::max(1, (waves + 3) / 4);
  p.iters = GPW;
  return p.res ? launch_kernel(pointwise_kernel<NT, KS, true>, dim3(grid), dim3(256), s, ev, p)
               : launch_kernel(pointwise_kernel<NT, KS, false>, dim3(grid), dim3(256), s, ev, p);
}

struct PwShape { int nt, ks; };
constexpr PwShape kPwShapes[] = {{6, 2}, {1, 12}, {1, 2}, {2, 2}, {4, 2}, {1, 4}, {2, 4}, {4, 4}, {1, 8}, {2, 8}};

bool pw_find(const OpLaunch& L, int* nt, int* ks) {
  if (L.op != LOP_CONV2D || L.dtype != LOP_BF16) return false;
  if (L.kh != 1 || L.kw != 1 || L.sh != 1 || L.sw != 1 || L.ph != 0 || L.pw != 0) return false;
  if (L.x.c % 16 != 0 || L.y.c % 32 != 0) return false;
  *nt = L.y.c / 32;
  *ks = L.x.c / 16;
  for (const PwShape& sh : kPwShapes)
    if (sh.nt == *nt && sh.ks == *ks) return true;
  return false;
}

}  // namespace

// True when the bandwidth-bound 1x1 kernel takes this launch instead of the implicit GEMM.
bool pointwise_applies(const OpLaunch& L) {
  int nt, ks;
  return pw_find(L, &nt, &ks);
}

int pointwise_describe(const OpLaunch& L, char* name, size_t size) {
  int nt = 0, ks = 0;
  pw_find(L, &nt, &ks);
  if (name && size)
    snprintf(name, size, "pointwise_kernel<%d, %d, %s>", nt, ks, L.res.ptr ? "true" : "false");
  return 1;
}

hipError_t launch_pointwise(const OpLaunch& L, hipStream_t stream, KernelEvents* ev) {
  int nt = 0, ks = 0;
  if (!pw_find(L, &nt, &ks)) return hipErrorInvalidValue;
  PwParams p;
  p.x = (const __bf16*)L.x.ptr; p.y = (__bf16*)L.y.ptr; p.res = (const __bf16*)L.res.ptr;
  p.w = (const __bf16*)L.w; p.bias = L.bias;
  p.x_row0 = L.x.row0; p.x_rows = L.x.rows; p.W = L.x.w; p.C_in = L.x.c;
  p.y_row0 = L.y.row0; p.y_rows = L.y.rows; p.C_out = L.y.c;
  p.r_row0 = L.res.row0; p.r_rows = L.res.rows;
  p.act = L.act; p.out_lo = L.out_lo; p.R = L.out_hi - L.out_lo; p.N = L.x.n;
  p.M = p.N * p.R * p.W;
  p.k_pad = L.k_pad;
  if (p.M <= 0) return hipSuccess;
  p.groups = (p.M + 31) / 32;
  p.iters = 0;
#define LOP_PW_CASE(NT, KS) if (nt == NT && ks == KS) return launch_pw<NT, KS>(p, stream, ev)
  LOP_PW_CASE(6, 2); LOP_PW_CASE(1, 12); LOP_PW_CASE(1, 2); LOP_PW_CASE(2, 2); LOP_PW_CASE(4, 2);
  LOP_PW_CASE(1, 4); LOP_PW_CASE(2, 4); LOP_PW_CASE(4, 4); LOP_PW_CASE(1, 8); LOP_PW_CASE(2, 8);
#undef LOP_PW_CASE
  return hipErrorInvalidValue;
}

}  // namespace lop
