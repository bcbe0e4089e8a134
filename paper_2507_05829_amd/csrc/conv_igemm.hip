// Dense convolution on a row interval as an implicit GEMM on the gfx950 matrix cores.
//
// GEMM view of the block-wise local operator (Intra-DP Sec. IV-A): rows are output
// pixels (n, oh, ow) with oh in the band's interval, columns are output channels, the
// reduction runs over k = (a*kw + b)*c_in + ci. Activations are NHWC so a run of
// channels of one tap is contiguous; the im2col matrix is never materialised: each
// workgroup gathers its K-slices (128 or 64 bytes per pixel and step) of BM pixels from the
// input slab through registers into LDS (zero where a tap falls outside the image; rows
// outside the slab are never needed by construction and are also taken as zero, and the
// load that stands in for them reads the slab's first bytes, so no access can leave the slab).
//
// Wave tiling: 4 wavefronts of 64 lanes (8 for the 256 x 256 tile), each owning TM x TN tiles of
// 32x32 (v_mfma_f32_32x32x16_bf16, or 4 x v_mfma_f32_32x32x2_f32 for fp32). The weight
// tile is the MFMA A operand and the pixel tile the B operand, so in the accumulator a
// lane holds 4 consecutive output channels of one pixel: bias, residual, activation and
// the single rounding to the storage type are applied in registers and stored as one
// vector per pixel.
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
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16 bytes in registers: a native vector, so that copies of it are loads and stores the
// optimiser can keep in registers (copies of HIP's uint4 struct are memcpy calls, and an
// array of them that is filled from memory stays in private memory)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Division of a pixel index by a width or a row count that only the host knows: q = (mulhi(n,
// mul) + n) >> shift for 0 <= n < 2^31 (Granlund and Montgomery's division by an invariant
// integer), three instructions where the integer division of two registers takes about forty,
// and a wavefront issues one instruction in four cycles or more.
struct FastDiv { unsigned mul; int shift; };
inline FastDiv make_fastdiv(int d) {
  FastDiv f{1u, 0};
  if (d < 1) return f;
  while ((1L << f.shift) < d) ++f.shift;
  f.mul = (unsigned)((((unsigned long long)1 << 32) * (((unsigned long long)1 << f.shift) - (unsigned long long)d)) / (unsigned long long)d + 1);
  return f;
}
__device__ __forceinline__ int fastdiv(int n, const FastDiv& f) {
  return (int)((__umulhi((unsigned)n, f.mul) + (unsigned)n) >> f.shift);
}

struct ConvParams {
  const void* x;
  void* y;
  void* y2;  // second destination with y's layout, or nullptr
  const void* res;
  const void* w;   // [c_out_pad][k_pad]
  const void* wd;  // the same weights in MFMA operand order (conv_direct_kernel), or nullptr
  const void* wd16;  // ... in the operand order of 16 x 16 tiles (conv_narrow_kernel), or nullptr
  const float* bias;
  float* ws;  // split-K partial sums [split][M][C_out], or nullptr
  int x_row0, x_rows, H, W, C_in;
  int y_row0, y_rows, W_out, C_out;
  int r_row0, r_rows;
  int kh, kw, sh, sw, ph, pw, dh, dw;
  int act, out_lo, R, N;
  int M;  // N * R * W_out
  int K, k_pad;
  int splits, kc_per_split;
  int pool;  // conv_lds_kernel<..., true>: R, out_lo, W_out and y describe the 2 x 2 max-pooled tensor
  FastDiv by_w, by_r;  // division by W_out and by R
  FastDiv by_group;    // ... by kGroupM x the launch's channel tiles (xcd_tile), set by the launchers that use it
};
static_assert(sizeof(Batch<ConvParams>) <= 4096, "the parameters of all bands of a launch travel as kernel arguments");

__device__ __forceinline__ float apply_act(float v, int act) {
  return clamp_act(v, make_clamp(act));
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float v) { return (__bf16)v; }

template <typename T>
__device__ __forceinline__ void mma(const u32x4& wa, const u32x4& px, f32x16& acc);

template <>
__device__ __forceinline__ void mma<__bf16>(const u32x4& wa, const u32x4& px, f32x16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa),
                                                __builtin_bit_cast(bf16x8, px), acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mma<float>(const u32x4& wa, const u32x4& px, f32x16& acc) {
  const f32x4 a = __builtin_bit_cast(f32x4, wa), b = __builtin_bit_cast(f32x4, px);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], acc, 0, 0, 0);
}

// LDS traffic inside one wavefront needs no barrier (the hardware keeps a wavefront's LDS
// instructions in issue order); only the compiler must not reorder a write and a later read
// of another lane's data.
__device__ __forceinline__ void lds_wave_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Output pixel m -> element offsets of its channel vector in y and in the residual.
struct PixelAddr {
  size_t y, r;
};
// Output pixel m of a launch -> image, row of the launch, column.
struct PixelAt { int n, r, ow; };
__device__ __forceinline__ PixelAt pixel_at(const ConvParams& p, int m) {
  PixelAt a;
  const int q = fastdiv(m, p.by_w);
  a.ow = m - q * p.W_out;
  a.n = fastdiv(q, p.by_r);
  a.r = q - a.n * p.R;
  return a;
}
__device__ __forceinline__ PixelAddr pixel_addr(const ConvParams& p, int m) {
  const PixelAt at = pixel_at(p, m);
  const int ow = at.ow, r = at.r, n = at.n;
  const int oh = p.out_lo + r;
  PixelAddr a;
  a.y = ((size_t)(n * p.y_rows + oh - p.y_row0) * p.W_out + ow) * p.C_out;
  a.r = p.res ? ((size_t)(n * p.r_rows + oh - p.r_row0) * p.W_out + ow) * p.C_out : 0;
  return a;
}

// bias + residual + activation + the one rounding, for 4 consecutive channels of a pixel.
template <typename T>
__device__ __forceinline__ void finish4(const ConvParams& p, const PixelAddr& a, int co, float* v) {
  T* __restrict__ yg = (T*)p.y;
  const T* __restrict__ rg = (const T*)p.res;
  if ((p.C_out & 3) == 0) {
    if (p.bias) {
      const float4 b4 = *(const float4*)(p.bias + co);
      v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
    }
    if (rg) {
      alignas(16) T rr[4];
      if (sizeof(T) == 2) *(uint2*)rr = *(const uint2*)(rg + a.r + co);
      else *(u32x4*)rr = *(const u32x4*)(rg + a.r + co);
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] += to_f32(rr[j]);
    }
    alignas(16) T o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = from_f32<T>(apply_act(v[j], p.act));
    if (sizeof(T) == 2) *(uint2*)(yg + a.y + co) = *(const uint2*)o;
    else *(u32x4*)(yg + a.y + co) = *(const u32x4*)o;
    if (p.y2) {
      if (sizeof(T) == 2) *(uint2*)((T*)p.y2 + a.y + co) = *(const uint2*)o;
      else *(u32x4*)((T*)p.y2 + a.y + co) = *(const u32x4*)o;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (co + j >= p.C_out) break;
      float u = v[j];
      if (p.bias) u += p.bias[co + j];
      if (rg) u += to_f32(rg[a.r + co + j]);
      const T o1 = from_f32<T>(apply_act(u, p.act));
      yg[a.y + co + j] = o1;
      if (p.y2) ((T*)p.y2)[a.y + co + j] = o1;
    }
  }
}

// bias + residual + activation + the one rounding for VE consecutive channels (one
// 16-byte vector of the storage type) of output pixel m.
template <typename T, int VE>
__device__ __forceinline__ void finish_vec(const ConvParams& p, int m, int co, float* v) {
  const PixelAddr pa = pixel_addr(p, m);
  if (p.bias) {
#pragma unroll
    for (int j = 0; j < VE; j += 4) {
      const float4 b4 = *(const float4*)(p.bias + co + j);
      v[j] += b4.x; v[j + 1] += b4.y; v[j + 2] += b4.z; v[j + 3] += b4.w;
    }
  }
  if (p.res) {
    alignas(16) T rr[VE];
    *(u32x4*)rr = *(const u32x4*)((const T*)p.res + pa.r + co);
#pragma unroll
    for (int j = 0; j < VE; ++j) v[j] += to_f32(rr[j]);
  }
  alignas(16) T o[VE];
#pragma unroll
  for (int j = 0; j < VE; ++j) o[j] = from_f32<T>(apply_act(v[j], p.act));
  *(u32x4*)((T*)p.y + pa.y + co) = *(const u32x4*)o;
  if (p.y2) *(u32x4*)((T*)p.y2 + pa.y + co) = *(const u32x4*)o;
}

// Which tile a workgroup takes. The hardware hands workgroups to the 8 XCDs round-robin in
// launch order (x fastest), and every XCD has an L2 of its own: in launch order the 64
// workgroups that are resident on one XCD at a time would be scattered over the whole grid
// and each would pull its own pixel tile and weight tile through that L2. Instead XCD k takes
// the k-th contiguous eighth of a walk over the tiles that goes down groups of kGroupM pixel
// tiles and then across the channel tiles, so its resident workgroups form a block of about
// 8 x 8 tiles that shares 8 pixel tiles and 8 weight tiles. Reduction slices are outermost.
struct TileId { int m, n, z; };
constexpr int kXcds = 8, kGroupM = 8;
// (by_group: division by kGroupM * ny, made on the host; the other divisions of this walk are by
// constants or lie behind conditions that hold for few workgroups)
__device__ __forceinline__ TileId xcd_tile(int bx, int mx, int ny, int nz, const FastDiv& by_group) {
  const int total = mx * ny * nz;
  const int launch = bx + mx * (blockIdx.y + ny * blockIdx.z);
  const int xcd = launch % kXcds, slot = launch / kXcds;
  const int q = total / kXcds, r = total % kXcds;
  const int v = xcd * q + min(xcd, r) + slot;  // XCD k owns q (+1 for the first r) consecutive tiles
  int z = 0, t = v;
  if (nz > 1) {
    const int per_z = mx * ny;
    z = v / per_z;
    t = v - z * per_z;
  }
  const int group = fastdiv(t, by_group), in_group = t - group * (kGroupM * ny);
  const int first = group * kGroupM;
  const int gm = min(kGroupM, mx - first);
  TileId id;
  id.z = z;
  id.n = gm == kGroupM ? in_group / kGroupM : in_group / gm;
  id.m = first + in_group - id.n * gm;
  return id;
}

// BM pixels x BN channels per workgroup; WM x WN wavefronts; BKB bytes of the reduction
// axis per row and step; VEC_A: c_in is a multiple of the 16-byte vector so one vector
// never straddles two taps. blockIdx.z selects a slice of the reduction (split-K): the
// slices' fp32 partial tiles go to p.ws and splitk_finish_kernel adds them in slice order.
template <typename T, int BM, int BN, int WM, int WN, int BKB, int NS, bool VEC_A>
__device__ __forceinline__ void conv_igemm_kernel_body(const ConvParams& p, const int bx, const int gx) {
  constexpr int KE = 16 / (int)sizeof(T);  // elements per 16-byte vector
  constexpr int CH = BKB / 16;             // vectors per row and step
  constexpr int BKE = CH * KE;             // reduction elements per step
  constexpr int ROWB = BKB + 16;           // LDS row pitch (16 pad bytes: conflict-free b128)
  constexpr int NW = WM * WN;              // wavefronts
  constexpr int RPP = 64 * NW / CH;        // rows filled per pass of all threads
  constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
  constexpr int A_IT = (BM + RPP - 1) / RPP, B_IT = (BN + RPP - 1) / RPP;
  static_assert((NW == 4 || NW == 8) && TM >= 1 && TN >= 1, "tile shape");

  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * (BM + BN) * ROWB];
  unsigned char* const As = smem;
  unsigned char* const Bs = smem + 2 * BM * ROWB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const TileId tile = xcd_tile(bx, gx, gridDim.y, gridDim.z, p.by_group);
  const int m0 = tile.m * BM, co0 = tile.n * BN;
  const int lrow = tid / CH, chunk = tid % CH;
  const T* __restrict__ xg = (const T*)p.x;
  const T* __restrict__ wg = (const T*)p.w;

  const int nk_all = p.k_pad / BKE;
  const int kc0 = tile.z * p.kc_per_split;
  const int kc1 = min(nk_all, kc0 + p.kc_per_split);

  // ---- the pixels this thread gathers (fixed over the K loop)
  int a_ih0[A_IT], a_iw0[A_IT], a_nrow[A_IT];
  int a_off[A_IT];
  bool a_ok[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = lrow + RPP * i;
    const int m = m0 + row;
    a_ok[i] = m < p.M && (BM % RPP == 0 || row < BM);
    const int mm = a_ok[i] ? m : 0;
    const PixelAt at = pixel_at(p, mm);
    const int ow = at.ow, r = at.r, n = at.n;
    a_ih0[i] = (p.out_lo + r) * p.sh - p.ph;
    a_iw0[i] = ow * p.sw - p.pw;
    a_nrow[i] = n * p.x_rows - p.x_row0;
    // element offset of tap (0, 0), channel 0 of this pixel (may lie before the slab: only
    // ever used together with a tap offset that the bounds check has accepted). 32 bits: the
    // host refuses a slab of 4 GiB or more, and so every load below is "uniform 64-bit base +
    // 32-bit per-thread byte offset", the cheapest form in registers and address arithmetic.
    a_off[i] = ((a_nrow[i] + a_ih0[i]) * p.W + a_iw0[i]) * p.C_in;
  }
  // rows of the packed weights this thread loads (never guarded: the packing is padded)
  // this thread's byte offset inside a group of RPP weight rows; the group and the step are
  // uniform and go into the base
  const unsigned b_voff = (unsigned)((lrow * p.k_pad + chunk * KE) * (int)sizeof(T));
  const int tap_row = p.dh * p.W * p.C_in, tap_col = p.dw * p.C_in;
  // position of this thread's vector inside the reduction axis (VEC_A path)
  int ci = 0, kwi = 0, khi = 0;
  if (VEC_A) {
    const int k = kc0 * BKE + chunk * KE;
    const int tap = k / p.C_in;
    ci = k - tap * p.C_in;
    khi = tap / p.kw;
    kwi = tap - khi * p.kw;
  }

  // NS steps of global loads in flight
  u32x4 ra0[A_IT], ra1[A_IT], ra2[A_IT], rb0[B_IT], rb1[B_IT], rb2[B_IT];

  // `okm` gets one bit per A vector: set when its tap lies inside the image and the slab.
  auto gather = [&](int kc, u32x4 (&ra)[A_IT], u32x4 (&rb)[B_IT], unsigned& okm) __attribute__((always_inline)) {
    okm = VEC_A ? 0u : ~0u;
    if (VEC_A) {
      // the tap's offset is the same for every pixel of this thread: one address add per load
      const int toff = khi * tap_row + kwi * tap_col + ci;
      const int dih = khi * p.dh, diw = kwi * p.dw;
      const bool tap_ok = khi < p.kh;
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        const int ih = a_ih0[i] + dih, iw = a_iw0[i] + diw;
        // (bitwise, not short-circuit: the test itself must not become a branch either)
        const bool ok = a_ok[i] & tap_ok & (ih >= p.x_row0) & (ih < p.x_row0 + p.x_rows) &
                        (iw >= 0) & (iw < p.W);
        // No branch around the load, and no use of its result here: a tap outside the image or
        // the slab reads the slab's first vector (always there) and is zeroed when the stage is
        // written to LDS. With the same number of loads on every path, and nothing consuming them
        // before that, the wait in front of a stage is "all but the two younger stages"; a
        // skipped load on some path, or a select right here, makes it "everything".
        const unsigned boff = (unsigned)((a_off[i] + toff) & -(int)ok) * (unsigned)sizeof(T);
        ra[i] = *(const u32x4*)((const unsigned char*)xg + boff);
        okm |= (unsigned)ok << i;
      }
      ci += BKE;
      while (ci >= p.C_in) {
        ci -= p.C_in;
        if (++kwi == p.kw) { kwi = 0; ++khi; }
      }
    } else {
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        alignas(16) T e[KE];
#pragma unroll
        for (int j = 0; j < KE; ++j) {
          const int k = kc * BKE + chunk * KE + j;
          const int tap = k / p.C_in, c = k - tap * p.C_in;
          const int a = tap / p.kw, b = tap - a * p.kw;
          const int ih = a_ih0[i] + a * p.dh, iw = a_iw0[i] + b * p.dw;
          const bool ok = a_ok[i] && k < p.K && ih >= p.x_row0 && ih < p.x_row0 + p.x_rows &&
                          iw >= 0 && iw < p.W;
          e[j] = ok ? xg[((size_t)(a_nrow[i] + ih) * p.W + iw) * p.C_in + c] : from_f32<T>(0.f);
        }
        ra[i] = *(const u32x4*)e;
      }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = lrow + RPP * i;
      const unsigned char* group = (const unsigned char*)(wg + ((size_t)(co0 + RPP * i) * p.k_pad + (size_t)kc * BKE));
      if (BN % RPP == 0 || row < BN) rb[i] = *(const u32x4*)(group + b_voff);
    }
  };
  auto stash = [&](int buf, const u32x4 (&ra)[A_IT], const u32x4 (&rb)[B_IT], unsigned okm) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int row = lrow + RPP * i;
      if (BM % RPP == 0 || row < BM)
        *(u32x4*)(As + (buf * BM + row) * ROWB + chunk * 16) = (okm >> i & 1u) ? ra[i] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = lrow + RPP * i;
      if (BN % RPP == 0 || row < BN) *(u32x4*)(Bs + (buf * BN + row) * ROWB + chunk * 16) = rb[i];
    }
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // Software pipeline: the global loads of NS steps are in flight in registers and one more
  // step sits in LDS; each step moves the oldest stage into the LDS buffer that is not being
  // read, refills its registers and multiplies. One barrier per step.
  // (every stage is a variable of its own and the step body is written out once per
  // stage: indexed through an array of stages they end up in private memory)
  static_assert(NS == 3, "the pipeline below is written out for three stages");
  unsigned ok0 = 0, ok1 = 0, ok2 = 0;
  auto multiply = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < BKB / 32; ++ks) {
      u32x4 px[TM], wt[TN];
      const int koff = ks * 32 + (lane >> 5) * 16;
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
        px[tm] = *(const u32x4*)(As + (buf * BM + (wm * TM + tm) * 32 + (lane & 31)) * ROWB + koff);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
        wt[tn] = *(const u32x4*)(Bs + (buf * BN + (wn * TN + tn) * 32 + (lane & 31)) * ROWB + koff);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) mma<T>(wt[tn], px[tm], acc[tn][tm]);
      // keep at most two sub-steps' fragments live: without this the LDS reads of all four are
      // hoisted to the top and the big tile no longer fits two workgroups' registers
      if (ks & 1) __builtin_amdgcn_sched_barrier(0);
    }
  };
  // One step: after the barrier the tile of this step is complete in LDS and nobody reads the
  // other buffer any more, so the next step's stage (RA, RB: loaded two steps ago) goes into
  // that buffer, its registers are refilled with the step NS further on, and the multiply of
  // this step runs over both: the LDS writes and the global loads sit in the shadow of the
  // MFMAs instead of in front of the barrier.
#define LOP_CONV_STEP(ST, RA, RB, OK)                               \
  if (kc + ST < kc1) {                                              \
    const int buf = (kc - kc0 + ST) & 1;                            \
    __syncthreads();                                                \
    if (kc + ST + 1 < kc1) {                                        \
      stash(buf ^ 1, RA, RB, OK);                                   \
      if (kc + ST + 1 + NS < kc1) gather(kc + ST + 1 + NS, RA, RB, OK); \
    }                                                               \
    multiply(buf);                                                  \
  }
#define LOP_CONV_STEP_FULL(ST, RA, RB, OK)                          \
  {                                                                 \
    const int buf = (kc - kc0 + ST) & 1;                            \
    __syncthreads();                                                \
    stash(buf ^ 1, RA, RB, OK);                                     \
    gather(kc + ST + 1 + NS, RA, RB, OK);                           \
    multiply(buf);                                                  \
  }
  int kc = kc0;
  if (VEC_A && kc0 + 2 * NS + 1 <= kc1) {
    // Steady state (vector gathers only; the element-wise gather of a narrow first layer has
    // one or two steps and its loads are conditional anyway): every step, its successor and
    // the refill NS beyond that exist. Nothing about the loads is conditional here, neither in
    // the loop nor on the way into it, which is what lets the wait in front of a stage leave
    // the two younger stages in flight.
    gather(kc0 + 0, ra0, rb0, ok0);
    gather(kc0 + 1, ra1, rb1, ok1);
    gather(kc0 + 2, ra2, rb2, ok2);
    stash(0, ra0, rb0, ok0);
    gather(kc0 + NS, ra0, rb0, ok0);
    for (; kc + 2 * NS + 1 <= kc1; kc += NS) {
      LOP_CONV_STEP_FULL(0, ra1, rb1, ok1)
      LOP_CONV_STEP_FULL(1, ra2, rb2, ok2)
      LOP_CONV_STEP_FULL(2, ra0, rb0, ok0)
    }
  } else {
    if (kc0 + 0 < kc1) gather(kc0 + 0, ra0, rb0, ok0);
    if (kc0 + 1 < kc1) gather(kc0 + 1, ra1, rb1, ok1);
    if (kc0 + 2 < kc1) gather(kc0 + 2, ra2, rb2, ok2);
    if (kc0 < kc1) {
      stash(0, ra0, rb0, ok0);
      if (kc0 + NS < kc1) gather(kc0 + NS, ra0, rb0, ok0);
    }
  }
  // the last steps (at most 2 * NS), each guarded; the stage named is the next step's
  for (; kc < kc1; kc += NS) {
    LOP_CONV_STEP(0, ra1, rb1, ok1)
    LOP_CONV_STEP(1, ra2, rb2, ok2)
    LOP_CONV_STEP(2, ra0, rb0, ok0)
  }
#undef LOP_CONV_STEP_FULL
#undef LOP_CONV_STEP

  // ---- epilogue. In the accumulator a lane holds, per 32x32 tile, pixel (lane & 31) and
  // channels g*8 + (lane >> 5)*4 + {0..3}, g = 0..3. The tile goes through LDS once so that
  // consecutive lanes then own consecutive 16-byte pieces of a pixel's channels: bias,
  // residual, activation and the one rounding are applied on whole vectors and every
  // store (and residual load) of a wavefront covers contiguous runs of memory.
  constexpr int VE = 16 / (int)sizeof(T);  // output elements per 16-byte store
  if (p.C_out % VE == 0) {
    // one wavefront stages one of its 32-pixel tiles at a time in a slot of its own: no
    // workgroup barrier beyond the first, and the slots need far less LDS than the K loop
    constexpr int CPW = TN * 32 + 4;  // fp32 pitch: conflict-free float4 rows
    static_assert(NW * 32 * CPW * 4 <= 2 * (BM + BN) * ROWB, "staging slots must fit the K-loop LDS");
    float* const Cw = (float*)smem + wave * (32 * CPW);
    __syncthreads();  // every wavefront is done reading the operand tiles
    constexpr int CPR = TN * 32 / VE;  // 16-byte pieces per pixel of the wavefront's tile
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      lds_wave_order();  // the previous tile's reads are issued before these writes
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(float4*)(Cw + (lane & 31) * CPW + tn * 32 + g * 8 + (lane >> 5) * 4) =
              make_float4(acc[tn][tm][g * 4], acc[tn][tm][g * 4 + 1], acc[tn][tm][g * 4 + 2],
                          acc[tn][tm][g * 4 + 3]);
      lds_wave_order();
#pragma unroll
      for (int slot = lane; slot < 32 * CPR; slot += 64) {
        const int row = slot / CPR, c = (slot % CPR) * VE;
        const int m = m0 + (wm * TM + tm) * 32 + row, co = co0 + wn * TN * 32 + c;
        if (m >= p.M || co >= p.C_out) continue;
        float v[VE];
#pragma unroll
        for (int j = 0; j < VE; j += 4) {
          const float4 t = *(const float4*)(Cw + row * CPW + c + j);
          v[j] = t.x; v[j + 1] = t.y; v[j + 2] = t.z; v[j + 3] = t.w;
        }
        if (p.ws) {
          float* dst = p.ws + ((size_t)tile.z * p.M + m) * p.C_out + co;
#pragma unroll
          for (int j = 0; j < VE; j += 4)
            *(float4*)(dst + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
          continue;
        }
        finish_vec<T, VE>(p, m, co, v);
      }
    }
    return;
  }
  // channel counts that are not a multiple of the vector: straight from the registers
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int m = m0 + (wm * TM + tm) * 32 + (lane & 31);
    if (m >= p.M) continue;
    PixelAddr pa;
    if (!p.ws) pa = pixel_addr(p, m);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int co = co0 + (wn * TN + tn) * 32 + g * 8 + (lane >> 5) * 4;
        if (co >= p.C_out) continue;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[tn][tm][g * 4 + j];
        if (p.ws) {
          float* dst = p.ws + ((size_t)tile.z * p.M + m) * p.C_out + co;
          if ((p.C_out & 3) == 0) {
            *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (co + j < p.C_out) dst[j] = v[j];
          }
        } else {
          finish4<T>(p, pa, co, v);
        }
      }
    }
  }
}

template <typename T, int BM, int BN, int WM, int WN, int BKB, int NS, bool VEC_A>
__global__ __launch_bounds__(64 * WM * WN) void conv_igemm_kernel(const ConvParams p) {
  conv_igemm_kernel_body<T, BM, BN, WM, WN, BKB, NS, VEC_A>(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
template <typename T, int BM, int BN, int WM, int WN, int BKB, int NS, bool VEC_A>
__global__ __launch_bounds__(64 * WM * WN) void conv_igemm_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_igemm_kernel_body<T, BM, BN, WM, WN, BKB, NS, VEC_A>(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}


// Adds the split-K slices in slice order and applies the epilogue: one thread per 4
// consecutive channels of a pixel.
template <typename T>
__device__ __forceinline__ void splitk_finish_kernel_body(const ConvParams& p, const int bx, const int gx) {
  const int cq = (p.C_out + 3) / 4;
  const long gid = (long)bx * 256 + threadIdx.x;
  if (gid >= (long)p.M * cq) return;
  const int m = (int)(gid / cq), co = (int)(gid % cq) * 4;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  const float* src = p.ws + (size_t)m * p.C_out + co;
  const size_t slice = (size_t)p.M * p.C_out;
  if ((p.C_out & 3) == 0) {
    constexpr int D = 8;  // loads in flight, added in slice order
    int s = 0;
    for (; s + D <= p.splits; s += D) {
      float4 t[D];
#pragma unroll
      for (int i = 0; i < D; ++i) t[i] = *(const float4*)(src + (s + i) * slice);
#pragma unroll
      for (int i = 0; i < D; ++i) {
        v[0] += t[i].x; v[1] += t[i].y; v[2] += t[i].z; v[3] += t[i].w;
      }
    }
    if (s < p.splits) {  // the last, partial group: slices past the end read as zero
      float4 t[D];
#pragma unroll
      for (int i = 0; i < D; ++i) {
        t[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s + i < p.splits) t[i] = *(const float4*)(src + (s + i) * slice);
      }
#pragma unroll
      for (int i = 0; i < D; ++i) {
        v[0] += t[i].x; v[1] += t[i].y; v[2] += t[i].z; v[3] += t[i].w;
      }
    }
  } else {
    for (int s = 0; s < p.splits; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (co + j < p.C_out) v[j] += src[s * slice + j];
  }
  finish4<T>(p, pixel_addr(p, m), co, v);
}

template <typename T>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const ConvParams p) {
  splitk_finish_kernel_body<T>(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
template <typename T>
__global__ __launch_bounds__(256) void splitk_finish_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  splitk_finish_kernel_body<T>(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}


// Small layers (few output pixels x channels, long reduction): one workgroup owns a
// 32-pixel x (32*NT)-channel tile and its WK wavefronts split the reduction axis among
// themselves, each taking one contiguous slice. Nothing is shared between the wavefronts
// during the reduction, so operands go straight from global memory into MFMA operand
// registers with no LDS staging and no barrier: per step a lane loads one 16-byte vector of
// activations and one of weights per channel tile, U steps in flight. The weights come from
// a second packing in operand order (p.wd: [channel tile of 32][step][lane] 16 bytes, lane =
// half*32 + channel, holding k = step*MK + half*KE ... + KE), so a wavefront's weight load
// is one contiguous KiB. What the epilogue needs (bias, residual, addresses) is loaded
// before the reduction starts, so the kernel has one round of memory latency per U steps
// plus one, not one more per epilogue operand. LDS is used once at the end to add the WK
// partial tiles in wavefront order and to hand each thread a contiguous 16-byte piece.
// With p.splits == 1 this replaces a split-K launch plus its finish kernel by one launch.
// Layers whose weights are too large for one workgroup per tile to stream (a compute unit
// sustains a small share of the HBM rate) also cut the reduction across blockIdx.z: every
// slice writes its fp32 partial tile to p.ws and splitk_finish_kernel adds the slices.
template <typename T, int WK, int NT>
__device__ __forceinline__ void conv_direct_kernel_body(const ConvParams& p, const int bx, const int gx) {
  constexpr int KE = 16 / (int)sizeof(T);  // elements per 16-byte vector
  constexpr int MK = 2 * KE;               // reduction elements per step (two lane halves)
  constexpr int U = (WK == 16 && NT == 2) ? 4 : 8;  // steps of loads in flight (register budget)
  constexpr int BM = 32, BN = 32 * NT;
  constexpr int CP = BN + 4;               // fp32 pitch of a staged partial tile
  constexpr int RW = WK < 8 ? WK : 8;      // partial tiles staged per round
  constexpr int VE = KE;
  constexpr int CPR = BN / VE;             // 16-byte pieces per pixel of the tile
  constexpr int SLOTS = BM * CPR;
  constexpr int SPT = (SLOTS + 64 * WK - 1) / (64 * WK);  // pieces per thread
  __shared__ __attribute__((aligned(16))) float part[RW][BM * CP];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int px = lane & 31, kg = lane >> 5;
  const int m0 = bx * BM, co0 = blockIdx.y * BN;
  const T* __restrict__ xg = (const T*)p.x;
  const u32x4* __restrict__ wg = (const u32x4*)p.wd;
  const bool partial = p.ws != nullptr;

  // ---- epilogue operands of this thread's pieces, in flight during the reduction
  bool e_ok[SPT];
  size_t e_y[SPT];
  int e_row[SPT], e_c[SPT];
  float e_bias[SPT][VE];
  u32x4 e_res[SPT];
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    const int slot = tid + s * 64 * WK;
    e_row[s] = slot / CPR;
    e_c[s] = (slot % CPR) * VE;
    const int mo = m0 + e_row[s], co = co0 + e_c[s];
    e_ok[s] = slot < SLOTS && mo < p.M && co < p.C_out;
    e_res[s] = u32x4{0u, 0u, 0u, 0u};
    e_y[s] = 0;
#pragma unroll
    for (int j = 0; j < VE; ++j) e_bias[s][j] = 0.f;
    if (e_ok[s] && partial) e_y[s] = ((size_t)blockIdx.z * p.M + mo) * p.C_out + co;
    if (e_ok[s] && !partial) {
      const PixelAddr pa = pixel_addr(p, mo);
      e_y[s] = pa.y + co;
      if (p.bias) {
#pragma unroll
        for (int j = 0; j < VE; j += 4) {
          const float4 b4 = *(const float4*)(p.bias + co + j);
          e_bias[s][j] = b4.x; e_bias[s][j + 1] = b4.y; e_bias[s][j + 2] = b4.z; e_bias[s][j + 3] = b4.w;
        }
      }
      if (p.res) e_res[s] = *(const u32x4*)((const T*)p.res + pa.r + co);
    }
  }

  // ---- this lane's pixel
  const int m = m0 + px;
  const bool m_ok = m < p.M;
  int ih0, iw0, nrow;
  {
    const int mm = m_ok ? m : 0;
    const PixelAt at = pixel_at(p, mm);
    const int ow = at.ow, r = at.r, n = at.n;
    ih0 = (p.out_lo + r) * p.sh - p.ph;
    iw0 = ow * p.sw - p.pw;
    nrow = n * p.x_rows - p.x_row0;
  }
  // this workgroup's slice of the reduction axis, then this wavefront's share of it, in
  // steps of MK elements
  const int steps_pad = p.k_pad / MK;         // pitch of the packed weights
  const int steps_all = (p.K + MK - 1) / MK;  // steps that hold anything
  const int z0 = blockIdx.z * p.kc_per_split, z1 = min(steps_all, z0 + p.kc_per_split);
  const int per_wave = (z1 - z0 + WK - 1) / WK;
  const int s0 = z0 + wave * per_wave, s1 = min(z1, s0 + per_wave);
  // position of this lane's vector on the reduction axis: k = (khi*kw + kwi)*C_in + ci
  int ci, kwi, khi;
  {
    const int k = s0 * MK + kg * KE;
    const int tap = k / p.C_in;
    ci = k - tap * p.C_in;
    khi = tap / p.kw;
    kwi = tap - khi * p.kw;
  }
  const u32x4* wtile[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
    wtile[t] = wg + (size_t)(blockIdx.y * NT + t) * steps_pad * 64 + lane;

  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

  for (int sb = s0; sb < s1; sb += U) {
    u32x4 a[U], w[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool live = sb + u < s1;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        w[u][t] = u32x4{0u, 0u, 0u, 0u};
        if (live) w[u][t] = wtile[t][(size_t)(sb + u) * 64];
      }
      const int ih = ih0 + khi * p.dh, iw = iw0 + kwi * p.dw;
      const bool ok = live && m_ok && khi < p.kh && ih >= p.x_row0 && ih < p.x_row0 + p.x_rows &&
                      iw >= 0 && iw < p.W;
      a[u] = u32x4{0u, 0u, 0u, 0u};
      if (ok) a[u] = *(const u32x4*)(xg + ((size_t)(nrow + ih) * p.W + iw) * p.C_in + ci);
      ci += MK;
      while (ci >= p.C_in) {
        ci -= p.C_in;
        if (++kwi == p.kw) { kwi = 0; ++khi; }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) mma<T>(w[u][t], a[u], acc[t]);
  }

  // ---- add the WK partial tiles in wavefront order, RW of them per round through LDS
  float v[SPT][VE];
#pragma unroll
  for (int s = 0; s < SPT; ++s)
#pragma unroll
    for (int j = 0; j < VE; ++j) v[s][j] = 0.f;
#pragma unroll
  for (int round = 0; round < WK / RW; ++round) {
    if (round) __syncthreads();  // the previous round's tiles have been read
    if (wave / RW == round) {
      float* const mine = part[wave % RW];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(float4*)(mine + px * CP + t * 32 + g * 8 + kg * 4) =
              make_float4(acc[t][g * 4], acc[t][g * 4 + 1], acc[t][g * 4 + 2], acc[t][g * 4 + 3]);
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < SPT; ++s) {
      if (!e_ok[s]) continue;
#pragma unroll
      for (int w = 0; w < RW; ++w)
#pragma unroll
        for (int j = 0; j < VE; j += 4) {
          const float4 q = *(const float4*)(&part[w][e_row[s] * CP + e_c[s] + j]);
          v[s][j] += q.x; v[s][j + 1] += q.y; v[s][j + 2] += q.z; v[s][j + 3] += q.w;
        }
    }
  }
  if (partial) {
#pragma unroll
    for (int s = 0; s < SPT; ++s) {
      if (!e_ok[s]) continue;
#pragma unroll
      for (int j = 0; j < VE; j += 4)
        *(float4*)(p.ws + e_y[s] + j) = make_float4(v[s][j], v[s][j + 1], v[s][j + 2], v[s][j + 3]);
    }
    return;
  }
  // ---- bias + residual + activation + the one rounding, one 16-byte store per piece
  const Clamp cl = make_clamp(p.act);
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    if (!e_ok[s]) continue;
    alignas(16) T rr[VE];
    *(u32x4*)rr = e_res[s];
    alignas(16) T o[VE];
#pragma unroll
    for (int j = 0; j < VE; ++j)
      o[j] = from_f32<T>(clamp_act(v[s][j] + e_bias[s][j] + to_f32(rr[j]), cl));
    *(u32x4*)((T*)p.y + e_y[s]) = *(const u32x4*)o;
    if (p.y2) *(u32x4*)((T*)p.y2 + e_y[s]) = *(const u32x4*)o;
  }
}

template <typename T, int WK, int NT>
__global__ __launch_bounds__(64 * WK) void conv_direct_kernel(const ConvParams p) {
  conv_direct_kernel_body<T, WK, NT>(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
template <typename T, int WK, int NT>
__global__ __launch_bounds__(64 * WK) void conv_direct_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_direct_kernel_body<T, WK, NT>(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}


// Mid-size layers (hundreds to tens of thousands of pixels, 64..512 channels, a reduction of
// hundreds to thousands of elements: most launches of the banded 224 x 224 and 720p chains).
// Such a launch is too small for the 128-wide tiles to cover the chip and too large for the
// operand-direct kernels, whose gathered 16-byte loads touch a new cache line per lane and
// whose 1024-thread workgroups hold a whole compute unit while they wait. Here a 256-thread
// workgroup owns a BM-pixel x BN-channel tile and both operands travel global -> LDS without
// passing through registers (global_load_lds, 16 bytes per lane): a wavefront's load covers 8
// rows (pixels of the im2col matrix, or output channels of the weights) x 128 contiguous bytes
// of the reduction axis, i.e. 8 whole cache lines, and NST - 1 stages of 128 bytes per row are
// in flight per workgroup without costing a register. The 16-byte chunks of a row are placed
// at chunk ^ (row & 7) inside the row's 128 bytes (the placement is chosen through the address
// each lane fetches from, since the LDS side of such a load is fixed: lane j writes bytes
// [16 j, 16 j + 16) of the instruction's KiB), so a wavefront's MFMA operand read - 32 rows,
// the same two chunks of each - hits every LDS bank equally. The four wavefronts split the
// reduction axis inside a stage (wavefront w multiplies the w-th quarter of the 128 bytes) and
// each accumulates the whole tile; the four partial tiles are added through LDS in wavefront
// order at the end, so no operand byte is read from LDS twice and the result does not depend
// on how the launch was cut. A tap outside the image (or the slab) is fetched from a
// zero-filled device array instead of being masked afterwards. Needs C_in * sizeof(T) to be a
// multiple of 128 (a stage lies inside one tap) or 64 (TPS below) and C_out a multiple of the
// 16-byte vector.
//
// POOL: a 2 x 2 stride-2 max pooling that follows the convolution is part of the launch. The
// rows of the tile are then the convolution's pixels in the order (image, pooled row, pooled
// column, position in the window), so every four consecutive rows are one window; the epilogue
// takes their maximum per channel before bias, activation and rounding (all three are
// non-decreasing, so the maximum of the rounded values is the rounded value of the maximum) and
// stores pooled pixels: the convolution's own output never exists in memory.
static __device__ __attribute__((aligned(256))) unsigned char g_zero_line[256];

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding
// and leaves the other counters alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
constexpr int vmcnt_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0xf << 8); }

//
// TPS: taps per stage. 1: C_in * sizeof(T) is a multiple of 128. 2: it is 64, a stage's 128
// bytes per row are two taps of 64 bytes (the lanes that fetch chunks 4..7 of a row address the
// second one), and the reduction axis may end in the middle of the last stage: the tap past the
// end is fetched from the zero line like a tap outside the image (its weights are zero padding).
template <typename T, int BM, int BN, int NST, bool POOL, int TPS>
__device__ __forceinline__ void conv_lds_kernel_body(const ConvParams& p, const int bx, const int gx) {
  constexpr int KE = 16 / (int)sizeof(T);   // elements per 16-byte chunk
  constexpr int SKE = 8 * KE;               // reduction elements per stage (128 bytes per row)
  constexpr int TM = BM / 32, TN = BN / 32; // 32 x 32 MFMA tiles of the workgroup tile
  constexpr int A_LD = BM / 32, B_LD = BN / 32;  // load instructions per wavefront and stage
  constexpr int LPS = A_LD + B_LD;
  constexpr int A_BYTES = BM * 128, STAGE = (BM + BN) * 128;
  constexpr int CP = BN + 4;                // fp32 pitch of a staged partial tile
  constexpr int VE = KE;
  constexpr bool AHEAD = sizeof(T) == 4;    // read the next stage's fragments during this stage's MFMAs
  constexpr int PIECES = BM * (BN / VE);    // 16-byte output pieces of the tile
  constexpr int RED_BYTES = 4 * BM * CP * 4;
  constexpr int SMEM = NST * STAGE > RED_BYTES ? NST * STAGE : RED_BYTES;
  static_assert(BM % 32 == 0 && BN % 32 == 0 && NST >= 3 && (NST - 2) * LPS < 64 && NST * STAGE <= 160 * 1024, "tile shape");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // every XCD takes a contiguous stretch of the tiles (a few pixel tiles times the channel
  // tiles), so that its L2 pulls a part of each operand instead of all of both
  const TileId tile = xcd_tile(bx, gx, gridDim.y, 1, p.by_group);
  const int m0 = tile.m * BM, co0 = tile.n * BN;
  const unsigned char* __restrict__ xg = (const unsigned char*)p.x;
  const unsigned char* __restrict__ wg = (const unsigned char*)p.w;
  const int ns = p.k_pad / SKE;             // stages

  // ---- what this lane fetches: row (lane >> 3) of an 8-row group, chunk (lane & 7) ^ row ^
  // (group & 1). A wavefront takes the groups wave, wave + 4, ..., which all have its parity.
  // (With the row alone as key, rows r and r + 8 of a fragment read share their banks where the
  // LDS serves 256 bytes per clock: the bank-conflict counter read 2.8-3.3 conflict cycles per
  // active LDS cycle, as much as a 4-way conflicting read pattern elsewhere.)
  const int lrow = lane >> 3;
  const int chunk = (lane & 7) ^ lrow ^ (wave & 1);
  constexpr int CPT = 8 / TPS;              // 16-byte chunks of one tap inside a stage
  const bool second = chunk >= CPT;         // TPS == 2: this lane fetches the stage's second tap
  int a_off[A_LD], a_ih0[A_LD], a_iw0[A_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    const int m = m0 + (wave + 4 * i) * 8 + lrow;
    const bool ok = m < p.M;
    const int mm = ok ? (POOL ? m >> 2 : m) : 0;
    const PixelAt at = pixel_at(p, mm);
    const int ow = at.ow, r = at.r, n = at.n;
    // the convolution's output pixel behind this row of the tile
    const int oy = POOL ? (p.out_lo + r) * 2 + ((m >> 1) & 1) : p.out_lo + r;
    const int ox = POOL ? ow * 2 + (m & 1) : ow;
    const int ih0 = oy * p.sh - p.ph, iw0 = ox * p.sw - p.pw;
    a_ih0[i] = ok ? ih0 : -(1 << 28);       // a row past the end of the launch: every tap "outside"
    a_iw0[i] = iw0;
    a_off[i] = (((n * p.x_rows - p.x_row0 + ih0) * p.W + iw0) * p.C_in + (chunk % CPT) * KE) * (int)sizeof(T);
  }
  unsigned b_off[B_LD];
#pragma unroll
  for (int i = 0; i < B_LD; ++i)
    b_off[i] = (unsigned)(((co0 + (wave + 4 * i) * 8 + lrow) * p.k_pad + chunk * KE) * (int)sizeof(T));
  const int tap_row = p.dh * p.W * p.C_in * (int)sizeof(T), tap_col = p.dw * p.C_in * (int)sizeof(T);

  // Workgroups that share an operand tile (the same pixels, or the same channels) would all ask
  // for the same cache lines at the same moment if they walked the reduction axis in step, and
  // the one that runs ahead would take every L2 miss of that tile by itself. Each workgroup
  // therefore starts at a stage of its own and wraps around: the first touches of a tile are
  // spread over the workgroups that share it. (The order of summation then depends on the tile
  // index; it is fixed for a given launch.)
  int st = (tile.m * 5 + tile.n * 11) % ns;
  // position of the next stage to issue on the reduction axis: k = (ia*kw + ib)*C_in + ici
  int ia, ib, ici, issued = 0;
  {
    const int k0 = st * SKE, tap = k0 / p.C_in;
    ici = k0 - tap * p.C_in;                // (TPS == 2: always 0)
    ia = tap / p.kw;
    ib = tap - ia * p.kw;
  }
  const unsigned char* const zero_src = g_zero_line + (lane & 7) * 16;  // what a padding tap fetches
  // One load instruction of the stage being issued: j < A_LD a pixel group, else a channel group.
  unsigned char* dst = smem;
  int toff = 0, dih = 0, diw = 0;
  bool tap_ok = true;
  unsigned koff = 0;
  auto issue_begin = [&]() __attribute__((always_inline)) {
    dst = smem + (issued % NST) * STAGE;
    if constexpr (TPS == 1) {
      toff = ia * tap_row + ib * tap_col + ici * (int)sizeof(T);
      dih = ia * p.dh;
      diw = ib * p.dw;
    } else {
      int ja = ia, jb = ib + 1;             // the stage's second tap
      if (jb == p.kw) { jb = 0; ++ja; }
      toff = second ? ja * tap_row + jb * tap_col : ia * tap_row + ib * tap_col;
      dih = (second ? ja : ia) * p.dh;
      diw = (second ? jb : ib) * p.dw;
      tap_ok = (second ? ja : ia) < p.kh;
    }
    koff = (unsigned)st * (unsigned)(SKE * (int)sizeof(T));
  };
  auto issue_one = [&](int j) __attribute__((always_inline)) {
    if (j < A_LD) {
      const int ih = a_ih0[j] + dih, iw = a_iw0[j] + diw;
      const bool ok = (ih >= p.x_row0) & (ih < p.x_row0 + p.x_rows) & (iw >= 0) & (iw < p.W) & tap_ok;
      const unsigned char* src = ok ? xg + (a_off[j] + toff) : zero_src;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(dst + (wave + 4 * j) * 1024),
                                       16, 0, 0);
    } else {
      const int i = j - A_LD;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(wg + b_off[i] + koff),
                                       (__attribute__((address_space(3))) void*)(dst + A_BYTES + (wave + 4 * i) * 1024),
                                       16, 0, 0);
    }
  };
  auto issue_end = [&]() __attribute__((always_inline)) {
    ++issued;
    if constexpr (TPS == 1) {
      ici += SKE;
      if (ici >= p.C_in) {
        ici = 0;
        if (++ib == p.kw) { ib = 0; ++ia; }
      }
    } else {
      ib += TPS;
      while (ib >= p.kw) { ib -= p.kw; ++ia; }
    }
    if (++st == ns) { st = 0; ia = 0; ib = 0; ici = 0; }
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // operand fragment of this lane inside a 32-row tile of a stage: row = lane & 31, chunks
  // 2 * wave + (lane >> 5)
  const int frow = lane & 31, fchunk = 2 * wave + (lane >> 5);
  const int foff = (frow >> 3) * 1024 + ((frow & 7) * 8 + (fchunk ^ (frow & 7) ^ ((frow >> 3) & 1))) * 16;
  // The operand reads are written as instructions: reads the compiler can see make it wait for
  // EVERY global -> LDS load in flight before each of them (it cannot tell which stage a read
  // touches), which would leave one stage in flight instead of NST - 1. The waits are placed by
  // hand instead: vmcnt before the barrier for the stage about to be read, lgkmcnt behind the
  // reads (tied to the fragment registers, so no MFMA can move in front of it).
  const unsigned lds0 = (unsigned)(unsigned long)(__attribute__((address_space(3))) unsigned char*)smem + foff;
  u32x4 px[TM], wt[TN];      // fragments of the stage being multiplied
  u32x4 px_n[TM], wt_n[TN];  // ... of the next stage, on their way from LDS meanwhile
  auto read_issue = [&](int s) __attribute__((always_inline)) {
    const unsigned at = lds0 + (unsigned)((s % NST) * STAGE);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(px_n[tm]) : "v"(at), "n"(tm * 4096) : "memory");
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(wt_n[tn]) : "v"(at), "n"(A_BYTES + tn * 4096) : "memory");
  };
  // waits for the reads of read_issue and makes the fragments current
  auto read_take = [&]() __attribute__((always_inline)) {
    if constexpr (TM == 2 && TN == 2)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(px_n[0]), "+v"(px_n[1]), "+v"(wt_n[0]), "+v"(wt_n[1]) :: "memory");
    else if constexpr (TM == 1 && TN == 2)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(px_n[0]), "+v"(wt_n[0]), "+v"(wt_n[1]) :: "memory");
    else if constexpr (TM == 2 && TN == 1)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(px_n[0]), "+v"(px_n[1]), "+v"(wt_n[0]) :: "memory");
    else {
      static_assert(TM == 1 && TN == 1, "tile shapes up to 64 x 64");
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(px_n[0]), "+v"(wt_n[0]) :: "memory");
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) px[tm] = px_n[tm];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) wt[tn] = wt_n[tn];
  };
  auto stage_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  // The MFMAs of the stage in the fragment registers, with the load instructions of a later stage
  // between them (LOADS: whether there is one to issue): a wavefront issues in order and a load
  // waits at issue until the memory pipeline takes it, so behind an MFMA that wait overlaps the
  // MFMA's execution instead of adding to it.
  auto multiply = [&](bool loads) __attribute__((always_inline)) {
    constexpr int NM = TM * TN;
    if (loads) issue_begin();
#pragma unroll
    for (int i = 0; i < (NM > LPS ? NM : LPS); ++i) {
      if (i < NM) {
        mma<T>(wt[i / TM], px[i % TM], acc[i / TM][i % TM]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (loads && i < LPS) {
        issue_one(i);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (loads) issue_end();
  };

  // ---- NST - 1 stages issued ahead; one barrier per stage. AHEAD (fp32, whose MFMAs of a stage
  // take four times as long as bf16's): behind the barrier of stage s the stage after it is
  // complete for every wavefront, its fragments are read from LDS while the MFMAs of stage s
  // run, and the loads issued among those MFMAs reuse the buffer of stage s - 1, which nobody
  // reads any more (+2.5 % on the fp32 chain). Otherwise the barrier follows the MFMAs and the
  // fragments of the next stage are read behind it (the bf16 loop is bound by what the L2s
  // deliver; reading ahead costs it one stage of prefetch depth and measured 2-3 % slower).
  const int pre = min(ns, NST - 1);
  for (int s = 0; s < pre; ++s) {
    issue_begin();
#pragma unroll
    for (int j = 0; j < LPS; ++j) issue_one(j);
    issue_end();
  }
  if (ns > NST - 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * LPS));
  else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  stage_barrier();
  read_issue(0);
  read_take();
  int s = 0;
  if constexpr (AHEAD) {
    for (; s + NST - 1 < ns; ++s) {  // stage s + NST - 1 is still to be issued (and stage s + 1 exists)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 3) * LPS));
      stage_barrier();
      read_issue(s + 1);
      multiply(true);
      read_take();
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    stage_barrier();                 // everything is in LDS, for every wavefront, and stays
    for (; s + 1 < ns; ++s) {
      read_issue(s + 1);
      multiply(false);
      read_take();
    }
  } else {
    for (; s + NST < ns; ++s) {      // stage s + NST - 1 exists and so does stage s + 1
      multiply(true);
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * LPS));
      stage_barrier();
      read_issue(s + 1);
      read_take();
    }
    if (s + NST - 1 < ns) {          // the last stage to issue
      multiply(true);
      ++s;
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      stage_barrier();
      read_issue(s);
      read_take();
    } else {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    for (; s + 1 < ns; ++s) {        // everything is in LDS (and stays: no barrier needed any more)
      multiply(false);
      read_issue(s + 1);
      read_take();
    }
  }
  multiply(false);

  // ---- add the four partial tiles in wavefront order through LDS, then the epilogue on
  // 16-byte pieces (a lane of the accumulator holds pixel lane & 31 and channels
  // g*8 + (lane >> 5)*4 + {0..3} of every 32 x 32 tile)
  __syncthreads();
  float* const mine = (float*)smem + wave * (BM * CP);
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *(float4*)(mine + (tm * 32 + (lane & 31)) * CP + tn * 32 + g * 8 + (lane >> 5) * 4) =
            make_float4(acc[tn][tm][g * 4], acc[tn][tm][g * 4 + 1], acc[tn][tm][g * 4 + 2], acc[tn][tm][g * 4 + 3]);
  __syncthreads();
  if constexpr (POOL) {
    for (int piece = tid; piece < PIECES / 4; piece += 256) {
      const int win = piece / (BN / VE), c = (piece % (BN / VE)) * VE;
      const int m = m0 + win * 4, co = co0 + c;
      if (m >= p.M || co >= p.C_out) continue;   // (M is a multiple of 4: whole windows)
      float best[VE];
#pragma unroll
      for (int turn = 0; turn < 4; ++turn) {
        // (neighbouring windows start at different positions of their window: four rows apart
        // they would read the same LDS banks at the same time)
        const int sub = (turn + win) & 3;
        float v[VE];
#pragma unroll
        for (int j = 0; j < VE; ++j) v[j] = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
          for (int j = 0; j < VE; j += 4) {
            const float4 q = *(const float4*)((const float*)smem + w * (BM * CP) + (win * 4 + sub) * CP + c + j);
            v[j] += q.x; v[j + 1] += q.y; v[j + 2] += q.z; v[j + 3] += q.w;
          }
#pragma unroll
        for (int j = 0; j < VE; ++j) best[j] = turn == 0 ? v[j] : fmaxf(best[j], v[j]);
      }
      finish_vec<T, VE>(p, m >> 2, co, best);
    }
    return;
  }
  for (int piece = tid; piece < PIECES; piece += 256) {
    const int row = piece / (BN / VE), c = (piece % (BN / VE)) * VE;
    const int m = m0 + row, co = co0 + c;
    if (m >= p.M || co >= p.C_out) continue;
    float v[VE];
#pragma unroll
    for (int j = 0; j < VE; ++j) v[j] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
      for (int j = 0; j < VE; j += 4) {
        const float4 q = *(const float4*)((const float*)smem + w * (BM * CP) + row * CP + c + j);
        v[j] += q.x; v[j + 1] += q.y; v[j + 2] += q.z; v[j + 3] += q.w;
      }
    finish_vec<T, VE>(p, m, co, v);
  }
}

template <typename T, int BM, int BN, int NST, bool POOL, int TPS>
__global__ __launch_bounds__(256) void conv_lds_kernel(const ConvParams p) {
  conv_lds_kernel_body<T, BM, BN, NST, POOL, TPS>(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
template <typename T, int BM, int BN, int NST, bool POOL, int TPS>
__global__ __launch_bounds__(256) void conv_lds_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_lds_kernel_body<T, BM, BN, NST, POOL, TPS>(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}


// Whether (and how) the direct kernel takes a launch: only layers that the tiled kernel
// would cut along the reduction axis, with vectorisable channel counts.
// 16 x 16 MFMA tiles of the same operand-direct scheme, for the layers with very few pixels
// and megabytes of weights (the last stages of a backbone once it is banded): a 16-pixel x
// 16-channel tile per workgroup gives four times as many workgroups as 32 x 32 tiles, enough to
// pull the whole weight tensor through the compute units' load paths in one launch, so the
// reduction need not be cut across workgroups and no finish kernel follows. Its 16 wavefronts
// split the reduction axis; weights come from a third packing ([channel tile of 16][step]
// [lane] 16 bytes, lane = quarter*16 + channel, holding k = step*MK + quarter*KE ... + KE,
// MK = 4 vectors), pixels straight from the input slab; the 16 partial tiles are added through
// LDS in wavefront order by the first wavefront, which also applies the epilogue.
template <typename T>
__device__ __forceinline__ void mma16(const u32x4& wa, const u32x4& px, f32x4& acc);
template <>
__device__ __forceinline__ void mma16<__bf16>(const u32x4& wa, const u32x4& px, f32x4& acc) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa),
                                                __builtin_bit_cast(bf16x8, px), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma16<float>(const u32x4& wa, const u32x4& px, f32x4& acc) {
  const f32x4 a = __builtin_bit_cast(f32x4, wa), b = __builtin_bit_cast(f32x4, px);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], acc, 0, 0, 0);
}

// Layers whose pixels are 64 bytes (32 bf16 channels in) under a 3 x 3 filter of horizontal
// stride 1 at hundreds of thousands of pixels: the second layer of the 720p chain when all its
// bands are one launch. The tiled kernels spend such a launch fetching: every workgroup pulls
// the taps of its pixels (nine times the layer's input) and the filter through the L2s for a
// reduction loop of five stages. Here a wavefront keeps the filter of 32 output channels in
// registers as MFMA operands (18 vectors of 16 bytes) and walks over tiles of 16 consecutive
// pixels of an input row; per tile and filter row it loads those 16 pixels once, straight into
// the other operand, multiplies them with each of the row's three filter columns into sums kept
// per column, and puts an output pixel together from the column sums of three neighbouring
// lanes: 14 output pixels per tile. No LDS, no barrier; the four wavefronts of a workgroup
// only share the filter's cache lines. Workgroups walk the tiles with a stride (XCD k over the k-th
// eighth of them, so that an XCD's L2 holds neighbouring image rows), which spreads the cost
// of loading the filter over several tiles. Measured on 856 000 pixels (32 -> 32 channels):
// 36 us against 91 us on the LDS-staged kernel (44 us in a form that loaded the two pixels
// behind a tile as well and shifted copies of the input between lanes). It is bound by the
// instructions around the 36 MFMAs of a round, not by memory (the loop with no load, store or
// MFMA in it takes two thirds of the time), so launches of one band (tens of thousands of
// pixels, where it measured no faster) stay on the LDS-staged kernel.
constexpr int kRegwTilePixels = 14;     // output pixels of a tile: 16 loaded pixels less the filter's two extra columns
constexpr int kRegwTiles = 8;           // tiles per workgroup and round: two per wavefront
constexpr int kRegwWorkgroups = 768;    // three per compute unit: all resident at once
constexpr int kRegwMinPixels = 1 << 17;

// rounds of workgroups it takes to cover a launch
__host__ __device__ inline int regw_groups(const ConvParams& p) {
  const int tiles = p.N * p.R * ((p.W_out + kRegwTilePixels - 1) / kRegwTilePixels);
  return (tiles + kRegwTiles - 1) / kRegwTiles;
}

__device__ __forceinline__ void conv_regw_kernel_body(const ConvParams& p, const int bx, const int gx) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // 16 x 16 x 32 MFMAs: lane (pxl, kq) holds channels 8 kq + {0..7} in of a pixel (or of an
  // output channel's filter tap), so the four lanes of a pixel read its 64 bytes together and a
  // wavefront's load covers 16 whole pixels
  const int pxl = lane & 15, kq = lane >> 4;
  const int co0 = blockIdx.y * 32;
  // The input slab as a buffer: a load whose offset lies beyond the buffer returns zeros without
  // touching memory, which is how a tap outside the image or the slab reads here (a select per
  // loaded register would cost as many instructions as the MFMAs take cycles).
  const __amdgpu_buffer_rsrc_t xbuf = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(p.x), 0, (int)((size_t)p.N * p.x_rows * p.W * 64), 0x00020000);
  constexpr unsigned kOutside = 0x80000000u;
  u32x4 wt[9][2];   // tap, half of the 32 output channels
  float bias[2][4];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int co = co0 + cb * 16;
    const unsigned char* wrow = (const unsigned char*)p.w + ((size_t)(co + pxl) * p.k_pad + kq * 8) * 2;
#pragma unroll
    for (int t = 0; t < 9; ++t) wt[t][cb] = *(const u32x4*)(wrow + t * 64);
    const float4 b4 = p.bias ? *(const float4*)(p.bias + co + kq * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    bias[cb][0] = b4.x; bias[cb][1] = b4.y; bias[cb][2] = b4.z; bias[cb][3] = b4.w;
  }
  const Clamp cl = make_clamp(p.act);
  // A tile is 14 consecutive pixels of ONE output row (16 loaded ones), so that image, row and
  // the three row offsets of a tile are the same for the whole wavefront (scalar arithmetic)
  // and a lane only adds its column; the last tile of a row may hang over its end. Eight tiles
  // per workgroup and round, two per wavefront.
  const int tpr = (p.W_out + kRegwTilePixels - 1) / kRegwTilePixels;
  const int groups = regw_groups(p);
  int grp = bx, step = gx, end = groups;
  if (gx % kXcds == 0) {   // (the hardware hands workgroups to the XCDs round-robin)
    const int per = (groups + kXcds - 1) / kXcds, xcd = bx % kXcds;
    grp = xcd * per + bx / kXcds;
    step = gx / kXcds;
    end = min(groups, (xcd + 1) * per);
  }
  // the tiles of this wavefront as (image, row of the launch, tile of the row), stepped from
  // round to round without a division; a tile past the end has an image index past the last
  int tcol[2], row[2], img[2];
#pragma unroll
  for (int tile = 0; tile < 2; ++tile) {
    const int t = grp * kRegwTiles + wave * 2 + tile;
    const int q = t / tpr;
    tcol[tile] = t - q * tpr;
    img[tile] = q / p.R;
    row[tile] = q - img[tile] * p.R;
  }
  const int adv = step * kRegwTiles;
  const int adv_q = adv / tpr, adv_col = adv - adv_q * tpr;
  const int adv_img = adv_q / p.R, adv_row = adv_q - adv_img * p.R;
  const int lane_in = (pxl - p.pw) * 64 + kq * 16;   // this lane's bytes in a row of the slab, from the tile's first column
  for (; grp < end; grp += step) {
    // Per tile and filter row ONE load: 16 consecutive pixels of the input row, the first of
    // them the first tap of the tile's first output pixel. Every filter column keeps sums of its
    // own over the three rows (the products of column b with the pixel a lane loaded), and
    // output pixel j is column 0's sum of lane j + column 1's of lane j + 1 + column 2's of lane
    // j + 2: two lane shifts per accumulator register instead of shifted copies of the input,
    // and 14 finished pixels per 16 loaded. A column outside the image loads as zeros like a
    // row outside. (The L1 hands a wavefront's 16-byte load over in about 33 cycles however its
    // lines hit: with nine loads per tile the kernel ran at the speed of that path.)
    u32x4 px[2][3];
    int ow[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      ow[tile] = tcol[tile] * kRegwTilePixels + pxl;
      const bool live = img[tile] < p.N;                       // (the same for the whole wavefront)
      const int ih0 = (p.out_lo + row[tile]) * p.sh - p.ph;    // (... and so are the rows of the taps)
      const int iw = ow[tile] - p.pw;                          // column of the pixel this lane loads
      const unsigned off_a = (iw >= 0) & (iw < p.W) ? (unsigned)(tcol[tile] * (kRegwTilePixels * 64) + lane_in) : kOutside;
#pragma unroll
      for (int a = 0; a < 3; ++a) {
        const int ih = ih0 + a * p.dh;
        const bool row_ok = live & (ih >= p.x_row0) & (ih < p.x_row0 + p.x_rows);
        const int row_base = row_ok ? ((img[tile] * p.x_rows - p.x_row0 + ih) * p.W) * 64 : 0;
        px[tile][a] = __builtin_amdgcn_raw_buffer_load_b128(xbuf, row_ok ? off_a : kOutside, row_base, 0);
      }
    }
    f32x4 acc[2][2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      f32x4 col[3][2];
#pragma unroll
      for (int b = 0; b < 3; ++b)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) col[b][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) mma16<__bf16>(wt[a * 3 + b][cb], px[tile][a], col[b][cb]);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          // (row_shl: lane j reads lane j + 1 / j + 2 of its row of 16; the last lanes read zero
          // and finish no pixel)
          // (the elements are copied out first: __builtin_bit_cast applied to an element of a
          // vector reads the vector's first element whatever the index)
          const float f1 = col[1][cb][i], f2 = col[2][cb][i];
          const float c1 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, f1), 0x101, 0xf, 0xf, true));
          const float c2 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, f2), 0x102, 0xf, 0xf, true));
          acc[tile][cb][i] = (col[0][cb][i] + c1) + c2;
        }
    }
    // bias + residual + activation + the one rounding: a lane holds channels
    // co0 + 16 cb + 4 kq + {0..3} of its pixel of either tile
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      if (img[tile] < p.N && pxl < kRegwTilePixels && ow[tile] < p.W_out) {
        const int oh = p.out_lo + row[tile];
        const long yrow = ((long)(img[tile] * p.y_rows + oh - p.y_row0) * p.W_out) * p.C_out + co0;
        const long rrow = p.res ? ((long)(img[tile] * p.r_rows + oh - p.r_row0) * p.W_out) * p.C_out + co0 : 0;
        const int in_row = ow[tile] * p.C_out + kq * 4;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          float v[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = acc[tile][cb][i] + bias[cb][i];
          if (p.res) {
            alignas(8) __bf16 rr[4];
            *(uint2*)rr = *(const uint2*)((const __bf16*)p.res + rrow + in_row + cb * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += (float)rr[i];
          }
          alignas(8) __bf16 o[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = (__bf16)clamp_act(v[i], cl);
          *(uint2*)((__bf16*)p.y + yrow + in_row + cb * 16) = *(const uint2*)o;
          if (p.y2) *(uint2*)((__bf16*)p.y2 + yrow + in_row + cb * 16) = *(const uint2*)o;
        }
      }
      // the same wavefront's tile of the next round
      tcol[tile] += adv_col;
      const int c1 = tcol[tile] >= tpr;
      tcol[tile] -= c1 ? tpr : 0;
      row[tile] += adv_row + c1;
      const int c2 = row[tile] >= p.R;
      row[tile] -= c2 ? p.R : 0;
      img[tile] += adv_img + c2;
    }
  }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void conv_regw_kernel(const ConvParams p) {
  conv_regw_kernel_body(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void conv_regw_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_regw_kernel_body(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}

// Whether the filter-in-registers kernel takes a launch (judged on all bands of a group together).
bool regw_applies(const ConvParams& p, int dtype) {
  if (dtype != LOP_BF16 || p.C_in != 32 || p.kh != 3 || p.kw != 3 || p.C_out % 32 != 0) return false;
  if (p.sw != 1 || p.dw != 1) return false;   // (a lane's taps are its neighbours' pixels)
  if (p.M < kRegwMinPixels || p.pool) return false;
  // 32-bit signed byte offsets into the input slab
  return (size_t)p.N * p.x_rows * p.W * p.C_in * 2 < ((size_t)1 << 31);
}

hipError_t launch_regw(const ConvParams* ps, int n, hipStream_t s, KernelEvents* ev) {
  const ConvParams& p = ps[0];
  const unsigned gy = (unsigned)(p.C_out / 32);
  long all = 0;
  for (int b = 0; b < n; ++b) all += regw_groups(ps[b]);
  if (all <= 0 || (int)gy * 32 > conv_cout_pad(p.C_out)) return hipErrorInvalidValue;
  // every band gets its share of the resident workgroups (a multiple of the XCD count, or all
  // of its pixel groups when those are fewer)
  unsigned gx[kMaxBatch];
  for (int b = 0; b < n; ++b) {
    if ((size_t)ps[b].N * ps[b].x_rows * ps[b].W * ps[b].C_in * 2 >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    const long groups = regw_groups(ps[b]);
    long share = (long)kRegwWorkgroups / gy * groups / all;
    share = share / kXcds * kXcds;
    gx[b] = (unsigned)(share >= kXcds && share < groups ? share : groups);
  }
  return launch_group(conv_regw_kernel, conv_regw_kernel_bands, ps, n, gx, gy, 1, dim3(256), s, ev);
}

constexpr int kNarrowWaves = 16;
// Stages of 128 bytes per row in LDS per workgroup. fp32: eight while the launch has at most one
// workgroup per compute unit (nothing else hides a workgroup's latency), four beyond that: with
// 64 KB per workgroup only two fit a compute unit, and a launch of several workgroups per unit
// runs a tenth faster when more of them are resident (the batched launches of the fp32 chain:
// 4 450 -> 4 920 images/s). bf16: four (three measured 3-6 % slower).
constexpr int kLdsStagesBf16 = 4, kLdsStagesF32 = 8, kLdsStagesF32Crowded = 4;
inline int f32_stages(long tiles) { return tiles > 256 ? kLdsStagesF32Crowded : kLdsStagesF32; }
constexpr long kLdsMaxLoopCycles = 25000;  // see lds_applies (40000 and 15000 measured: the fp32 chain gains down to 15000, the bf16 chains lose below 25000)
constexpr long kLdsOverTiledMaxTiles = 4 * 256;   // see lds_applies (2 048 and more measured slower than the tiled kernel)
constexpr int kLdsMinTiles = 48;   // below this the operand-direct kernels (one round of latency) win; 96 and 20 measured slower

template <typename T>
__device__ __forceinline__ void conv_narrow_kernel_body(const ConvParams& p, const int bx, const int gx) {
  constexpr int WK = kNarrowWaves;
  constexpr int KE = 16 / (int)sizeof(T);  // elements per 16-byte vector
  constexpr int MK = 4 * KE;               // reduction elements per step (four lane quarters)
  constexpr int U = 8;                     // steps of loads in flight
  constexpr int CP = 20;                   // fp32 pitch of a staged 16 x 16 partial tile
  constexpr int VE = KE;
  constexpr int CPR = 16 / VE;             // 16-byte pieces per pixel of the tile
  constexpr int SLOTS = 16 * CPR;          // <= 64: the first wavefront finishes the tile
  __shared__ __attribute__((aligned(16))) float part[WK][16 * CP];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int px = lane & 15, kq = lane >> 4;
  const int m0 = bx * 16, co0 = blockIdx.y * 16;
  const T* __restrict__ xg = (const T*)p.x;
  const u32x4* __restrict__ wg = (const u32x4*)p.wd16;

  // ---- epilogue operands of the finishing lanes, in flight during the reduction
  const int e_row = tid / CPR, e_c = (tid % CPR) * VE;
  const bool e_ok = tid < SLOTS && m0 + e_row < p.M && co0 + e_c < p.C_out;
  size_t e_y = 0;
  float e_bias[VE];
  u32x4 e_res = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < VE; ++j) e_bias[j] = 0.f;
  if (e_ok) {
    const int co = co0 + e_c;
    const PixelAddr pa = pixel_addr(p, m0 + e_row);
    e_y = pa.y + co;
    if (p.bias) {
#pragma unroll
      for (int j = 0; j < VE; j += 4) {
        const float4 b4 = *(const float4*)(p.bias + co + j);
        e_bias[j] = b4.x; e_bias[j + 1] = b4.y; e_bias[j + 2] = b4.z; e_bias[j + 3] = b4.w;
      }
    }
    if (p.res) e_res = *(const u32x4*)((const T*)p.res + pa.r + co);
  }

  // ---- this lane's pixel
  const int m = m0 + px;
  const bool m_ok = m < p.M;
  int ih0, iw0, nrow;
  {
    const int mm = m_ok ? m : 0;
    const PixelAt at = pixel_at(p, mm);
    const int ow = at.ow, r = at.r, n = at.n;
    ih0 = (p.out_lo + r) * p.sh - p.ph;
    iw0 = ow * p.sw - p.pw;
    nrow = n * p.x_rows - p.x_row0;
  }
  const int steps_pad = p.k_pad / MK;         // pitch of the packed weights
  const int steps_all = (p.K + MK - 1) / MK;  // steps that hold anything
  const int per_wave = (steps_all + WK - 1) / WK;
  const int s0 = wave * per_wave, s1 = min(steps_all, s0 + per_wave);
  int ci, kwi, khi;  // position of this lane's vector: k = (khi*kw + kwi)*C_in + ci
  {
    const int k = s0 * MK + kq * KE;
    const int tap = k / p.C_in;
    ci = k - tap * p.C_in;
    khi = tap / p.kw;
    kwi = tap - khi * p.kw;
  }
  const u32x4* const wtile = wg + (size_t)blockIdx.y * steps_pad * 64 + lane;

  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int sb = s0; sb < s1; sb += U) {
    u32x4 a[U], w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool live = sb + u < s1;
      w[u] = u32x4{0u, 0u, 0u, 0u};
      if (live) w[u] = wtile[(size_t)(sb + u) * 64];
      const int ih = ih0 + khi * p.dh, iw = iw0 + kwi * p.dw;
      const bool ok = live && m_ok && khi < p.kh && ih >= p.x_row0 && ih < p.x_row0 + p.x_rows &&
                      iw >= 0 && iw < p.W;
      a[u] = u32x4{0u, 0u, 0u, 0u};
      if (ok) a[u] = *(const u32x4*)(xg + ((size_t)(nrow + ih) * p.W + iw) * p.C_in + ci);
      ci += MK;
      while (ci >= p.C_in) {
        ci -= p.C_in;
        if (++kwi == p.kw) { kwi = 0; ++khi; }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) mma16<T>(w[u], a[u], acc);
  }

  // ---- in the accumulator a lane holds channels kq*4 + {0..3} of pixel px
  *(float4*)(part[wave] + px * CP + kq * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  __syncthreads();
  if (!e_ok) return;
  float v[VE];
#pragma unroll
  for (int j = 0; j < VE; ++j) v[j] = 0.f;
#pragma unroll
  for (int w = 0; w < WK; ++w)
#pragma unroll
    for (int j = 0; j < VE; j += 4) {
      const float4 q = *(const float4*)(&part[w][e_row * CP + e_c + j]);
      v[j] += q.x; v[j + 1] += q.y; v[j + 2] += q.z; v[j + 3] += q.w;
    }
  const Clamp cl = make_clamp(p.act);
  alignas(16) T rr[VE];
  *(u32x4*)rr = e_res;
  alignas(16) T o[VE];
#pragma unroll
  for (int j = 0; j < VE; ++j) o[j] = from_f32<T>(clamp_act(v[j] + e_bias[j] + to_f32(rr[j]), cl));
  *(u32x4*)((T*)p.y + e_y) = *(const u32x4*)o;
  if (p.y2) *(u32x4*)((T*)p.y2 + e_y) = *(const u32x4*)o;
}

template <typename T>
__global__ __launch_bounds__(64 * kNarrowWaves) void conv_narrow_kernel(const ConvParams p) {
  conv_narrow_kernel_body<T>(p, blockIdx.x, gridDim.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1] of x).
template <typename T>
__global__ __launch_bounds__(64 * kNarrowWaves) void conv_narrow_kernel_bands(const Batch<ConvParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_narrow_kernel_body<T>(t.p[b], blockIdx.x - t.first[b], t.first[b + 1] - t.first[b]);
}


constexpr int kComputeUnits = 256;
constexpr int kNarrowMaxTiles = 320;

// The LDS-staged mid-size kernel: which tile, or bm == 0 when it does not apply.
struct LdsChoice { int bm, bn; long tiles; };
// The tile of a launch. The reduction loop of this kernel is bound by the rate at which one
// compute unit pulls its tile's operand rows (BM + BN rows of 128 bytes per stage), and launches
// of this size leave compute units idle: a smaller tile spreads the same rows over more compute
// units, until there are more workgroups than units and some unit has to take two. So the cost of
// a shape is (workgroups per compute unit, rounded up) x (BM + BN); the cheapest shape with at
// least min_tiles workgroups wins, the larger one on a tie (less traffic from the L2s).
LdsChoice pick_lds_tile(const ConvParams& p, int dtype, long min_tiles) {
  auto tiles = [&](int bm, int bn) { return (long)((p.M + bm - 1) / bm) * ((p.C_out + bn - 1) / bn); };
  if (dtype != LOP_BF16) return tiles(32, 32) >= min_tiles ? LdsChoice{32, 32, tiles(32, 32)} : LdsChoice{0, 0, 0};
  static const int shapes[][2] = {{64, 64}, {32, 64}, {64, 32}, {32, 32}};
  LdsChoice best{0, 0, 0};
  long best_cost = 0;
  for (const auto& sh : shapes) {
    if (sh[1] == 32 && sh[0] == 64 && p.C_out > 32) continue;   // (the 64 x 32 tile is there for narrow layers)
    const long t = tiles(sh[0], sh[1]);
    if (t < min_tiles) continue;
    const long cost = (t + kComputeUnits - 1) / kComputeUnits * (sh[0] + sh[1]);
    if (!best.bm || cost < best_cost) { best = {sh[0], sh[1], t}; best_cost = cost; }
  }
  return best;
}

LdsChoice choose_lds(const ConvParams& p, int dtype) {
  const int esz = dtype == LOP_BF16 ? 2 : 4, ke = 16 / esz;
  const bool half_rows = p.C_in * esz == 64;   // two taps per stage
  if (!half_rows && ((p.C_in * esz) % 128 != 0 || p.k_pad != p.K)) return {0, 0, 0};
  if (p.C_out % ke != 0 || (p.k_pad * esz) % 128 != 0) return {0, 0, 0};
  // 32-bit signed byte offsets into the input slab
  if ((size_t)p.N * p.x_rows * p.W * p.C_in * esz >= ((size_t)1 << 31)) return {0, 0, 0};
  return pick_lds_tile(p, dtype, kLdsMinTiles);
}

// blocks of x per band for tiles of `per` pixels
inline void blocks_per_band(const ConvParams* ps, int n, int per, unsigned* gx) {
  for (int b = 0; b < n; ++b) gx[b] = (unsigned)((ps[b].M + per - 1) / per);
}

// Copies of the bands' parameters that know the launch's channel-tile count (xcd_tile's divisor).
inline void with_tile_walk(const ConvParams* ps, int n, unsigned gy, ConvParams* out) {
  for (int b = 0; b < n; ++b) {
    out[b] = ps[b];
    out[b].by_group = make_fastdiv(kGroupM * (int)gy);
  }
}

template <typename T, int BM, int BN, int NST>
hipError_t launch_lds(const ConvParams* ps_in, int n, hipStream_t s, KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  const ConvParams& p = ps_in[0];
  unsigned gx[kMaxBatch];
  blocks_per_band(ps_in, n, BM, gx);
  const unsigned gy = (unsigned)((p.C_out + BN - 1) / BN);
  if ((int)gy * BN > conv_cout_pad(p.C_out)) return hipErrorInvalidValue;
  ConvParams ps[kMaxBatch];
  with_tile_walk(ps_in, n, gy, ps);
  const int row_bytes = p.C_in * (int)sizeof(T);
  if (row_bytes == 64) {
    if (p.pool) return hipErrorInvalidValue;
    return launch_group(conv_lds_kernel<T, BM, BN, NST, false, 2>, conv_lds_kernel_bands<T, BM, BN, NST, false, 2>,
                        ps, n, gx, gy, 1, dim3(256), s, ev);
  }
  if (row_bytes % 128 != 0 || p.k_pad != p.K) return hipErrorInvalidValue;
  if (p.pool)
    return launch_group(conv_lds_kernel<T, BM, BN, NST, true, 1>, conv_lds_kernel_bands<T, BM, BN, NST, true, 1>,
                        ps, n, gx, gy, 1, dim3(256), s, ev);
  return launch_group(conv_lds_kernel<T, BM, BN, NST, false, 1>, conv_lds_kernel_bands<T, BM, BN, NST, false, 1>,
                      ps, n, gx, gy, 1, dim3(256), s, ev);
}

struct DirectChoice {
  int wk, nt;      // wk == 0: not applicable
  int z, per_z;    // slices of the reduction across workgroups, steps per slice
  bool narrow = false;  // conv_narrow_kernel (16 x 16 tiles, one launch) instead
};
DirectChoice choose_direct(const ConvParams& p, int dtype, int splits) {
  const int ke = dtype == LOP_BF16 ? 8 : 4;
  // (also layers whose tile grid is a fraction of the chip even without a cut: they are
  // latency-bound, and this kernel has fewer rounds of latency)
  const long tiles = (long)((p.M + 31) / 32) * ((p.C_out + 31) / 32);
  if (!p.wd || (splits <= 1 && tiles > kComputeUnits) || p.C_in % ke != 0 || p.C_out % ke != 0) return {0, 0, 0, 0};
  const int steps = (p.K + 2 * ke - 1) / (2 * ke);
  const long mt32 = (p.M + 31) / 32, nt32 = (p.C_out + 31) / 32;
  // one workgroup per tile streams steps KiB of weights and as much of activations, and
  // fp32 MFMA runs at 1/16 of the bf16 rate: beyond these lengths the reduction is cut
  const int single_max = dtype == LOP_BF16 ? 256 : 128;
  DirectChoice d{4, 1, 1, steps};
  if (steps <= single_max) {
    if (p.C_out > 32 && mt32 * nt32 >= 512) d.nt = 2;  // plenty of workgroups anyway
    while (d.wk < 16 && (steps + d.wk - 1) / d.wk > 8) d.wk *= 2;
    return d;
  }
  // at most two rounds of loads per wavefront and about one workgroup per compute unit: 16 x 16
  // tiles finish the layer in one launch, as fast as the cut and its finish kernel together
  // (measured 12 against 8 + 4 us on 560 pixels x 128 channels, 7 against 6 + 4 on 196 x 256)
  // and one launch fewer on the stream; with more tiles than that the workgroups (1024 threads,
  // one per compute unit) come in rounds, with a longer reduction the tiles' own latency chain
  // and, in fp32, MFMA time exceed the cut's
  const int steps16 = (p.K + 4 * ke - 1) / (4 * ke);
  const long tiles16 = (long)((p.M + 15) / 16) * ((p.C_out + 15) / 16);
  if (p.wd16 && tiles16 <= kNarrowMaxTiles && steps16 <= 16 * kNarrowWaves) {
    d.narrow = true;
    d.z = 1;
    return d;
  }
  // a slice is one round of loads per wavefront (4 wavefronts x 8 steps)
  d.z = std::min(64, (steps + 31) / 32);
  d.per_z = (steps + d.z - 1) / d.z;
  d.z = (steps + d.per_z - 1) / d.per_z;
  return d;
}

template <typename T, int WK, int NT>
hipError_t launch_direct(const ConvParams* ps, int n, hipStream_t s, KernelEvents* ev) {
  const ConvParams& p = ps[0];
  unsigned gx[kMaxBatch];
  blocks_per_band(ps, n, 32, gx);
  const unsigned gy = (unsigned)((p.C_out + 32 * NT - 1) / (32 * NT));
  if ((int)gy * 32 * NT > conv_cout_pad(p.C_out)) return hipErrorInvalidValue;  // unguarded weight loads
  return launch_group(conv_direct_kernel<T, WK, NT>, conv_direct_kernel_bands<T, WK, NT>, ps, n, gx, gy,
                      (unsigned)p.splits, dim3(64 * WK), s, ev);
}

template <typename T>
hipError_t launch_direct_any(const ConvParams* ps, int n, const DirectChoice& d, hipStream_t s,
                             KernelEvents* ev) {
  if (d.narrow) {
    unsigned gx[kMaxBatch];
    blocks_per_band(ps, n, 16, gx);
    const unsigned gy = (unsigned)((ps[0].C_out + 15) / 16);
    if ((int)gy * 16 > conv_cout_pad(ps[0].C_out)) return hipErrorInvalidValue;
    return launch_group(conv_narrow_kernel<T>, conv_narrow_kernel_bands<T>, ps, n, gx, gy, 1,
                        dim3(64 * kNarrowWaves), s, ev);
  }
  if (d.nt == 2) {
    if (d.wk == 4) return launch_direct<T, 4, 2>(ps, n, s, ev);
    if (d.wk == 8) return launch_direct<T, 8, 2>(ps, n, s, ev);
    return launch_direct<T, 16, 2>(ps, n, s, ev);
  }
  if (d.wk == 4) return launch_direct<T, 4, 1>(ps, n, s, ev);
  if (d.wk == 8) return launch_direct<T, 8, 1>(ps, n, s, ev);
  return launch_direct<T, 16, 1>(ps, n, s, ev);
}

enum Shape { S128x128, S128x64, S64x64, S128x32, S256x256 };
struct Choice {
  Shape shape;
  int bm, bn;
  int splits, kc_per_split;
};

constexpr int kBKB = 128;       // bytes of the reduction axis per row and step
constexpr int kBigBKB = 64;     // ... of the 256 x 256 tile (its registers and LDS allow no more)
constexpr int kStages = 3;      // steps of global loads kept in flight

// The 256 x 256 tile (eight wavefronts of 128 x 64, one workgroup per compute unit) moves half
// the operand bytes per multiply-add of the 128 x 128 tile and reads LDS three times for every
// four MFMAs instead of four times: measured a fifth faster per unit of tile area. But the chip
// holds 256 of them at a time against 512 of the smaller tile, so the last, partly filled round
// of workgroups weighs more. With t the time a compute unit needs for its two concurrent
// 128 x 128 tiles, a round of the big tile (four tile areas) takes 4 / 2 / 1.2 = 5/3 t.
bool big_tile_pays(long blocks256, long blocks128) {
  const long rounds256 = (blocks256 + kComputeUnits - 1) / kComputeUnits;
  const long rounds128 = (blocks128 + 2 * kComputeUnits - 1) / (2 * kComputeUnits);
  return rounds256 * 5 < rounds128 * 3;
}

// Largest tile that still gives every compute unit a workgroup; layers too small for
// that take the smallest tile and cut the reduction axis into slices until the grid
// covers the chip about twice (each slice keeps at least 4 steps).
Choice choose(const ConvParams& p, int dtype) {
  auto blocks = [&](int bm, int bn) {
    return (long)((p.M + bm - 1) / bm) * ((p.C_out + bn - 1) / bn);
  };
  Choice c;
  constexpr int kKE16 = 8;  // bf16 elements per 16-byte vector
  if (dtype == LOP_BF16 && p.C_out > kConvCoutPad && p.C_in % kKE16 == 0 && p.C_out % kKE16 == 0 &&
      blocks(256, 256) >= kComputeUnits &&
      big_tile_pays(blocks(256, 256), blocks(128, 128))) {
    c = {S256x256, 256, 256, 1, p.k_pad / (kBigBKB / 2)};
    return c;
  }
  if (p.C_out > 64 && blocks(128, 128) >= kComputeUnits) c = {S128x128, 128, 128, 1, 0};
  else if (p.C_out > 32 && blocks(128, 64) >= kComputeUnits) c = {S128x64, 128, 64, 1, 0};
  else if (p.C_out > 32) c = {S64x64, 64, 64, 1, 0};
  else c = {S128x32, 128, 32, 1, 0};
  const int bke = kBKB / (dtype == LOP_BF16 ? 2 : 4);
  const int nk = p.k_pad / bke;
  const long b = blocks(c.bm, c.bn);
  int splits = 1;
  if (b < kComputeUnits) {
    splits = (int)((2 * kComputeUnits + b - 1) / b);
    splits = std::min(splits, std::max(nk / 4, 1));
    splits = std::min(splits, 64);
  }
  c.kc_per_split = (nk + splits - 1) / splits;
  c.splits = (nk + c.kc_per_split - 1) / c.kc_per_split;
  return c;
}

// The mid-size kernel takes a launch that the operand-direct kernels would otherwise take
// (the tiled kernel keeps the layers large enough for its 128-wide tiles to cover the chip)
// unless the 16 x 16-tile kernel finishes it in one round of workgroups.
LdsChoice lds_applies(const ConvParams& p, int dtype, const Choice& c, const DirectChoice& d) {
  if (c.shape == S256x256) return {0, 0, 0};
  if (c.splits == 1 && (c.shape == S128x128 || c.shape == S128x64)) {
    // (a layer that just covers the chip with 128-wide tiles: up to four rounds of this kernel's
    // tiles it is still the faster one - 256 -> 256 channels on 9 800 pixels 34 against 39 us)
    const LdsChoice few = choose_lds(p, dtype);
    return few.bm && few.tiles <= kLdsOverTiledMaxTiles ? few : LdsChoice{0, 0, 0};
  }
  if (d.wk && d.narrow) return {0, 0, 0};
  const LdsChoice ld = choose_lds(p, dtype);
  // A workgroup of this kernel walks the whole reduction axis by itself, pulling BM + BN rows of
  // 128 bytes per stage at what one compute unit gets from the L2s (about 25 bytes per clock). A
  // layer of few pixels and a long reduction (512 -> 512 channels at 7 x 7) leaves most compute
  // units idle while the few walk for tens of microseconds: cutting the reduction across
  // workgroups (the operand-direct kernel and its finish kernel) is faster there.
  if (ld.bm && ld.tiles < kComputeUnits && d.wk && d.z > 1) {
    const long stages = (long)p.k_pad * (dtype == LOP_BF16 ? 2 : 4) / 128;
    if (stages * (ld.bm + ld.bn) * 128 / 25 > kLdsMaxLoopCycles) return {0, 0, 0};
  }
  return ld;
}

template <typename T>
hipError_t launch_finish(const ConvParams* ps, int n, hipStream_t s, KernelEvents* ev) {
  unsigned gx[kMaxBatch];
  for (int b = 0; b < n; ++b) gx[b] = (unsigned)(((long)ps[b].M * ((ps[b].C_out + 3) / 4) + 255) / 256);
  return launch_group(splitk_finish_kernel<T>, splitk_finish_kernel_bands<T>, ps, n, gx, 1, 1, dim3(256), s, ev);
}

template <typename T, int BM, int BN, int WM, int WN>
hipError_t launch_shape(const ConvParams* ps_in, int n, bool vec_a, hipStream_t s, KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  const ConvParams& p = ps_in[0];
  unsigned gx[kMaxBatch];
  blocks_per_band(ps_in, n, BM, gx);
  const unsigned gy = (unsigned)((p.C_out + BN - 1) / BN);
  ConvParams ps[kMaxBatch];
  with_tile_walk(ps_in, n, gy, ps);
  const dim3 block(64 * WM * WN);
  // weight loads are unguarded: the channel tiles must end inside the padded packing
  if ((int)gy * BN > conv_cout_pad(p.C_out)) return hipErrorInvalidValue;
  const hipError_t e =
      vec_a ? launch_group(conv_igemm_kernel<T, BM, BN, WM, WN, kBKB, kStages, true>,
                           conv_igemm_kernel_bands<T, BM, BN, WM, WN, kBKB, kStages, true>, ps, n, gx, gy,
                           (unsigned)p.splits, block, s, ev)
            : launch_group(conv_igemm_kernel<T, BM, BN, WM, WN, kBKB, kStages, false>,
                           conv_igemm_kernel_bands<T, BM, BN, WM, WN, kBKB, kStages, false>, ps, n, gx, gy,
                           (unsigned)p.splits, block, s, ev);
  if (e != hipSuccess || !p.ws) return e;
  return launch_finish<T>(ps, n, s, ev);
}

// The parameters a group of bands is judged by when a kernel is chosen for all of them: those
// of the first band with the pixels of all (every other field that matters is the layer's).
ConvParams group_params(const ConvParams* ps, int n) {
  ConvParams g = ps[0];
  for (int b = 1; b < n; ++b) g.M += ps[b].M;
  return g;
}

// Whether the filter-in-registers kernel takes a group of bands: the layer and the group's
// pixels qualify and every band's slab is within reach of its 32-bit offsets.
bool regw_takes(const ConvParams* ps, int n, int dtype) {
  if (!regw_applies(group_params(ps, n), dtype)) return false;
  for (int b = 0; b < n; ++b)
    if ((size_t)ps[b].N * ps[b].x_rows * ps[b].W * ps[b].C_in * 2 >= ((size_t)1 << 31)) return false;
  return true;
}

// Split-K partial sums of the bands of a group, one region after the other in the workspace.
size_t assign_workspace(ConvParams* ps, int n, int splits, int kc_per_split, float* ws) {
  size_t at = 0;
  for (int b = 0; b < n; ++b) {
    ps[b].splits = splits;
    ps[b].kc_per_split = kc_per_split;
    ps[b].ws = splits > 1 && ws ? ws + at : nullptr;
    if (splits > 1) at += (size_t)splits * ps[b].M * ps[b].C_out;
  }
  return at * sizeof(float);
}

template <typename T>
hipError_t launch_typed(ConvParams* ps, int n, int dtype, float* ws, hipStream_t s, KernelEvents* ev) {
  constexpr int KE = 16 / (int)sizeof(T);
  const bool vec_a = ps[0].C_in % KE == 0;
  // the kernels address a slab with 32-bit byte offsets
  for (int b = 0; b < n; ++b)
    if ((size_t)ps[b].N * ps[b].x_rows * ps[b].W * ps[b].C_in * sizeof(T) >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  const ConvParams g = group_params(ps, n);
  if constexpr (sizeof(T) == 2) {
    if (regw_takes(ps, n, dtype)) {
      for (int b = 0; b < n; ++b) ps[b].ws = nullptr;
      return launch_regw(ps, n, s, ev);
    }
  }
  const Choice c = choose(g, dtype);
  const DirectChoice d = choose_direct(g, dtype, c.splits);
  const LdsChoice ld = lds_applies(g, dtype, c, d);
  if (ld.bm) {
    for (int b = 0; b < n; ++b) {
      ps[b].ws = nullptr;
      if ((size_t)ps[b].N * ps[b].x_rows * ps[b].W * ps[b].C_in * sizeof(T) >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    }
    if constexpr (sizeof(T) == 2) {
      // (twice the stages in flight, 128 KB of LDS, measured no faster per launch - the loop is
      // bound by what the L2s deliver, not by latency - and it keeps other streams' workgroups
      // off the compute unit)
      if (ld.bm == 32 && ld.bn == 32) return launch_lds<T, 32, 32, kLdsStagesBf16>(ps, n, s, ev);
      if (ld.bn == 32) return launch_lds<T, 64, 32, kLdsStagesBf16>(ps, n, s, ev);
      if (ld.bm == 64) return launch_lds<T, 64, 64, kLdsStagesBf16>(ps, n, s, ev);
      return launch_lds<T, 32, 64, kLdsStagesBf16>(ps, n, s, ev);
    } else {
      if (f32_stages(ld.tiles) == kLdsStagesF32Crowded) return launch_lds<T, 32, 32, kLdsStagesF32Crowded>(ps, n, s, ev);
      return launch_lds<T, 32, 32, kLdsStagesF32>(ps, n, s, ev);
    }
  }
  if (d.wk) {
    if (d.z > 1 && !ws) return hipErrorInvalidValue;
    assign_workspace(ps, n, d.z, d.per_z, ws);
    const hipError_t e = launch_direct_any<T>(ps, n, d, s, ev);
    if (e != hipSuccess || !ps[0].ws) return e;
    return launch_finish<T>(ps, n, s, ev);
  }
  if (c.splits > 1 && !ws) return hipErrorInvalidValue;
  assign_workspace(ps, n, c.splits, c.kc_per_split, ws);
  if (c.shape == S256x256) {
    if constexpr (sizeof(T) == 2) {
      if (n != 1) return hipErrorInvalidValue;   // (chosen for single launches of at least 256 tiles only)
      dim3 grid((ps[0].M + 255) / 256, (ps[0].C_out + 255) / 256, 1);
      ConvParams p;
      with_tile_walk(ps, 1, grid.y, &p);
      if ((int)grid.y * 256 > conv_cout_pad(p.C_out)) return hipErrorInvalidValue;
      return launch_kernel(conv_igemm_kernel<T, 256, 256, 2, 4, kBigBKB, kStages, true>, grid, dim3(512), s, ev, p);
    }
    return hipErrorInvalidValue;
  }
  switch (c.shape) {
    case S128x128: return launch_shape<T, 128, 128, 2, 2>(ps, n, vec_a, s, ev);
    case S128x64: return launch_shape<T, 128, 64, 2, 2>(ps, n, vec_a, s, ev);
    case S64x64: return launch_shape<T, 64, 64, 2, 2>(ps, n, vec_a, s, ev);
    default: return launch_shape<T, 128, 32, 4, 1>(ps, n, vec_a, s, ev);
  }
}

ConvParams make_params(const OpLaunch& L) {
  ConvParams p;
  p.x = L.x.ptr; p.y = L.y.ptr; p.y2 = L.y2; p.res = L.res.ptr; p.w = L.w; p.wd = L.wd; p.wd16 = L.wd16; p.bias = L.bias;
  p.ws = nullptr;
  p.x_row0 = L.x.row0; p.x_rows = L.x.rows; p.H = L.x.h; p.W = L.x.w; p.C_in = L.x.c;
  p.y_row0 = L.y.row0; p.y_rows = L.y.rows; p.W_out = L.y.w; p.C_out = L.y.c;
  p.r_row0 = L.res.row0; p.r_rows = L.res.rows;
  p.kh = L.kh; p.kw = L.kw; p.sh = L.sh; p.sw = L.sw; p.ph = L.ph; p.pw = L.pw;
  p.dh = L.dh; p.dw = L.dw;
  p.act = L.act; p.out_lo = L.out_lo; p.R = L.out_hi - L.out_lo; p.N = L.x.n;
  p.M = p.N * p.R * p.W_out;
  p.by_w = make_fastdiv(p.W_out);
  p.by_r = make_fastdiv(p.R);
  p.by_group = make_fastdiv(1);
  p.K = L.x.c * L.kh * L.kw;
  p.k_pad = L.k_pad;
  p.splits = 1;
  p.kc_per_split = 0;
  p.pool = 0;
  return p;
}

}  // namespace

int conv_k_pad(int c_in, int kh, int kw, int dtype) {
  const int bke = kBKB / (dtype == LOP_BF16 ? 2 : 4);
  const int k = c_in * kh * kw;
  return (k + bke - 1) / bke * bke;
}

namespace {
// Parameters of the bands of a group that compute something (n_out of them).
int group_of(const OpLaunch* Ls, int n, ConvParams* ps) {
  int m = 0;
  for (int b = 0; b < n && m < kMaxBatch; ++b) {
    const ConvParams p = make_params(Ls[b]);
    if (p.M > 0) ps[m++] = p;
  }
  return m;
}
}  // namespace

size_t conv_workspace_bytes_bands(const OpLaunch* Ls, int n) {
  if (n < 1 || n > kMaxBatch || stem_applies(Ls[0])) return 0;
  ConvParams ps[kMaxBatch];
  const int m = group_of(Ls, n, ps);
  if (m == 0) return 0;
  const int dtype = Ls[0].dtype;
  const ConvParams g = group_params(ps, m);
  if (regw_takes(ps, m, dtype)) return 0;
  const Choice c = choose(g, dtype);
  const DirectChoice d = choose_direct(g, dtype, c.splits);
  if (lds_applies(g, dtype, c, d).bm) return 0;
  if (d.wk) return d.z > 1 ? assign_workspace(ps, m, d.z, d.per_z, nullptr) : 0;
  return c.splits > 1 ? assign_workspace(ps, m, c.splits, c.kc_per_split, nullptr) : 0;
}

size_t conv_workspace_bytes(const OpLaunch& L) { return conv_workspace_bytes_bands(&L, 1); }

hipError_t launch_conv_igemm_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  ConvParams ps[kMaxBatch];
  const int m = group_of(Ls, n, ps);
  if (m == 0) return hipSuccess;
  return Ls[0].dtype == LOP_BF16 ? launch_typed<__bf16>(ps, m, Ls[0].dtype, (float*)Ls[0].ws, stream, ev)
                                 : launch_typed<float>(ps, m, Ls[0].dtype, (float*)Ls[0].ws, stream, ev);
}

hipError_t launch_conv_igemm(const OpLaunch& L, hipStream_t stream, KernelEvents* ev) {
  return launch_conv_igemm_bands(&L, 1, stream, ev);
}

// Name of the kernel instance as a profiler prints it, and the number of K slices.
int conv_igemm_describe_bands(const OpLaunch* Ls, int n, char* name, size_t size) {
  ConvParams ps[kMaxBatch];
  const int m = n >= 1 && n <= kMaxBatch ? group_of(Ls, n, ps) : 0;
  if (m == 0) {
    if (name && size) name[0] = 0;
    return 0;
  }
  const OpLaunch& L = Ls[0];
  const ConvParams p = group_params(ps, m);
  const char* const form = m > 1 ? "_bands" : "";
  const bool bf = L.dtype == LOP_BF16;
  const bool vec = p.C_in % (bf ? 8 : 4) == 0;
  if (regw_takes(ps, m, L.dtype)) {
    if (name && size) snprintf(name, size, "conv_regw_kernel%s", form);
    return 1;
  }
  const Choice c = choose(p, L.dtype);
  static const int wm[] = {2, 2, 2, 4, 2}, wn[] = {2, 2, 2, 1, 4};
  const DirectChoice d = choose_direct(p, L.dtype, c.splits);
  if (const LdsChoice ld = lds_applies(p, L.dtype, c, d); ld.bm) {
    if (name && size)
      snprintf(name, size, "conv_lds_kernel%s<%s, %d, %d, %d, false, %d>", form, bf ? "__bf16" : "float", ld.bm, ld.bn,
               bf ? kLdsStagesBf16 : f32_stages(ld.tiles), p.C_in * (bf ? 2 : 4) == 64 ? 2 : 1);
    return 1;
  }
  if (d.wk) {
    if (name && size) {
      if (d.narrow) snprintf(name, size, "conv_narrow_kernel%s<%s>", form, bf ? "__bf16" : "float");
      else snprintf(name, size, "conv_direct_kernel%s<%s, %d, %d>", form, bf ? "__bf16" : "float", d.wk, d.nt);
    }
    return d.z;
  }
  if (name && size)
    snprintf(name, size, "conv_igemm_kernel%s<%s, %d, %d, %d, %d, %d, %d, %s>", form, bf ? "__bf16" : "float",
             c.bm, c.bn, wm[c.shape], wn[c.shape], c.shape == S256x256 ? kBigBKB : kBKB, kStages,
             vec ? "true" : "false");
  return c.splits;
}

int conv_igemm_describe(const OpLaunch& L, char* name, size_t size) {
  if (make_params(L).M <= 0) {   // (a band that computes nothing of the layer still names its kernel)
    OpLaunch one = L;
    one.out_hi = one.out_lo + 1;
    return conv_igemm_describe_bands(&one, 1, name, size);
  }
  return conv_igemm_describe_bands(&L, 1, name, size);
}

// ---- convolution + the 2 x 2 stride-2 max pooling behind it as one launch (conv_lds_kernel<..., true>)

namespace {
// Parameters of the pooled launch: the convolution's operands and hyper-parameters with the
// pooled tensor's rows, width and slab as the output.
ConvParams make_pooled_params(const OpLaunch& conv, const OpLaunch& pool) {
  OpLaunch o = conv;
  o.y = pool.y;
  o.y2 = pool.y2;
  o.out_lo = pool.out_lo;
  o.out_hi = pool.out_hi;
  ConvParams p = make_params(o);
  p.pool = 1;
  p.M *= 4;
  return p;
}
// The tile of a pooled launch: the LDS kernel always takes it (there is no other kernel that
// pools), with the smaller pixel tile when the larger would leave most of the chip idle.
LdsChoice choose_pooled(const ConvParams& p, int dtype) {
  const LdsChoice c = pick_lds_tile(p, dtype, 1);
  return c.bm ? c : LdsChoice{32, 32, 1};
}
}  // namespace

bool convpool_applies(const OpLaunch& conv, const OpLaunch& pool) {
  if (conv.op != LOP_CONV2D || pool.op != LOP_MAXPOOL2D || conv.res.ptr) return false;
  if (pool.kh != 2 || pool.kw != 2 || pool.sh != 2 || pool.sw != 2 || pool.ph != 0 || pool.pw != 0 ||
      pool.dh != 1 || pool.dw != 1)
    return false;
  const int esz = conv.dtype == LOP_BF16 ? 2 : 4, ke = 16 / esz;
  const int K = conv.x.c * conv.kh * conv.kw;
  return (conv.x.c * esz) % 128 == 0 && conv.y.c % ke == 0 && conv.k_pad == K;
}

// Whether the pooled launch is worth taking for this launch of the conv (its own rows, its
// slabs' geometry): not where the conv alone would run on one of the operand-direct kernels
// (few pixels, a long reduction), which together with a separate pooling launch are faster
// than the LDS kernel on so few tiles (8 + 4 us against 15-17 us on the 512-channel layers of
// a banded VGG-16).
bool convpool_pays(const OpLaunch& conv) {
  const ConvParams p = make_params(conv);
  if (p.M <= 0) return true;
  const Choice c = choose(p, conv.dtype);
  const DirectChoice d = choose_direct(p, conv.dtype, c.splits);
  return !(d.wk && d.narrow);
}

hipError_t launch_convpool_bands(const OpLaunch* convs, const OpLaunch* pools, int n, hipStream_t stream,
                                 KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  ConvParams ps[kMaxBatch];
  int m = 0;
  const int esz = convs[0].dtype == LOP_BF16 ? 2 : 4;
  for (int b = 0; b < n; ++b) {
    const ConvParams p = make_pooled_params(convs[b], pools[b]);
    if (p.M <= 0) continue;
    if (!convpool_applies(convs[b], pools[b])) return hipErrorInvalidValue;
    // 32-bit signed byte offsets into the input slab
    if ((size_t)p.N * p.x_rows * p.W * p.C_in * esz >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    ps[m++] = p;
  }
  if (m == 0) return hipSuccess;
  const LdsChoice ld = choose_pooled(group_params(ps, m), convs[0].dtype);
  if (convs[0].dtype == LOP_BF16) {
    if (ld.bm == 32 && ld.bn == 32) return launch_lds<__bf16, 32, 32, kLdsStagesBf16>(ps, m, stream, ev);
    if (ld.bn == 32) return launch_lds<__bf16, 64, 32, kLdsStagesBf16>(ps, m, stream, ev);
    if (ld.bm == 64) return launch_lds<__bf16, 64, 64, kLdsStagesBf16>(ps, m, stream, ev);
    return launch_lds<__bf16, 32, 64, kLdsStagesBf16>(ps, m, stream, ev);
  }
  if (f32_stages(ld.tiles) == kLdsStagesF32Crowded) return launch_lds<float, 32, 32, kLdsStagesF32Crowded>(ps, m, stream, ev);
  return launch_lds<float, 32, 32, kLdsStagesF32>(ps, m, stream, ev);
}

hipError_t launch_convpool(const OpLaunch& conv, const OpLaunch& pool, hipStream_t stream, KernelEvents* ev) {
  return launch_convpool_bands(&conv, &pool, 1, stream, ev);
}

int convpool_describe_bands(const OpLaunch* convs, const OpLaunch* pools, int n, char* name, size_t size) {
  ConvParams ps[kMaxBatch];
  int m = 0;
  for (int b = 0; b < n && m < kMaxBatch; ++b) {
    const ConvParams p = make_pooled_params(convs[b], pools[b]);
    if (p.M > 0) ps[m++] = p;
  }
  if (m == 0) {
    if (name && size) name[0] = 0;
    return 0;
  }
  const LdsChoice ld = choose_pooled(group_params(ps, m), convs[0].dtype);
  const bool bf = convs[0].dtype == LOP_BF16;
  if (name && size)
    snprintf(name, size, "conv_lds_kernel%s<%s, %d, %d, %d, true, 1>", m > 1 ? "_bands" : "", bf ? "__bf16" : "float",
             ld.bm, ld.bn, bf ? kLdsStagesBf16 : f32_stages(ld.tiles));
  return 1;
}

int convpool_describe(const OpLaunch& conv, const OpLaunch& pool, char* name, size_t size) {
  return convpool_describe_bands(&conv, &pool, 1, name, size);
}

}  // namespace lop
