// First layers of a backbone: a dense convolution over very few input channels (an RGB image),
// e.g. 7 x 7 stride 2 over 3 channels. The reduction axis is short (27 .. 192 elements) and does
// not come in 16-byte pieces (3 channels), so the implicit-GEMM kernels gather it element by
// element; the arithmetic itself is small enough for the vector ALUs (Sec. IV-A local operator:
// every output pixel depends on a kh x kw window of the input only).
//
// Two forms. For launches of thousands of 64-pixel tiles (conv_stem_lane_kernel): a lane owns one
// output pixel and CPL (16 or 32) output channels, a wavefront 64 consecutive pixels of one
// output row. The lane loads the kw * C_in contiguous elements of every row of its window itself
// (neighbouring lanes read overlapping bytes: the L1 serves them) and, for every element of the
// reduction axis, multiplies it into its CPL accumulators with weights whose address is the same
// for the whole wavefront (the compiler turns those loads into scalar loads, and the
// multiply-adds take the weights from scalar registers). The weights are packed
// [C_out / 16][K][16] fp32 for that, behind the [C_out / 4][K][4] packing of the other form. No
// LDS and no barrier: at these sizes the other form spends more time launching its tens of
// thousands of workgroups and waiting for their one batch of loads than computing. For smaller
// launches (conv_stem_kernel, further down) the window of 64 pixels is staged in LDS and four
// wavefronts share its pixels. KJ: kw * C_in when it is one of the usual values (the loop over
// a kernel row is then unrolled), else 0.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>

#include "act.hpp"
#include "kernels.hpp"
#include "launch.hpp"
#include "lop.h"

namespace lop {
namespace {

constexpr int kStemPixels = 64;       // output pixels per wavefront (one per lane)
constexpr int kStemChannels = 16;     // output channels per packed weight group
constexpr int kStemPatchMax = 4096;   // fp32 elements of the staged input patch
constexpr int kStemRowChunks = 3;     // a staged row has at most 3 * 256 elements
constexpr int kStemLaneMinWaves = 4096;  // four per SIMD: below, the LDS-staged form (at 3 600 wavefronts it measured 23 us against 25)
constexpr int kStemMaxCin = 4;
constexpr int kStemMaxK = 192;

struct StemParams {
  const void* x;
  void* y;
  void* y2;             // second destination with y's layout, or nullptr
  const float* wq;      // [C_out / 4][K][4] (the LDS-staged form)
  const float* wq16;    // [C_out / 16][K][16] (the lane-owned form), behind the former
  const float* bias;    // or nullptr
  int x_row0, x_rows, W, C_in;
  int y_row0, y_rows, W_out, C_out;
  int kh, kw, sh, sw, ph, pw;
  int act, out_lo, R, N;
  int tiles_x;          // 64-pixel tiles per output row
  int patch_w;          // elements of one staged input row: ((64 - 1) * sw + kw) * C_in
};

__device__ __forceinline__ float load_f32(const float* p) { return *p; }
__device__ __forceinline__ float load_f32(const __bf16* p) { return (float)*p; }
// n consecutive channels (a multiple of 8) of one pixel
template <int N>
__device__ __forceinline__ void store_run(float* y, const float* v) {
#pragma unroll
  for (int j = 0; j < N; j += 4) *(float4*)(y + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
}
template <int N>
__device__ __forceinline__ void store_run(__bf16* y, const float* v) {
#pragma unroll
  for (int j = 0; j < N; j += 8) {
    alignas(16) __bf16 o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)v[j + i];
    *(uint4*)(y + j) = *(const uint4*)o;
  }
}

template <typename T, int KJ, int CPL>
__device__ __forceinline__ void conv_stem_lane_kernel_body(const StemParams& p, const int bx) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tile = bx * 4 + wave;                       // (the same for the whole wavefront)
  if (tile >= p.tiles_x * p.R * p.N) return;
  const int xt = tile % p.tiles_x;
  const int t = tile / p.tiles_x;
  const int r = t % p.R, n = t / p.R;
  const int oy = p.out_lo + r, ox = xt * kStemPixels + lane;
  const bool lane_ok = ox < p.W_out;
  const int ih0 = oy * p.sh - p.ph;
  const int e0 = (ox * p.sw - p.pw) * p.C_in;           // first element of the window in its row; may be negative
  const int row_elems = p.W * p.C_in;
  const int kj = KJ ? KJ : p.kw * p.C_in;               // reduction elements per kernel row
  const T* const xg = (const T*)p.x + (size_t)n * p.x_rows * row_elems;
  constexpr int G = CPL / kStemChannels;                // packed weight groups of this lane's channels
  const float* wq = p.wq16 + (size_t)(blockIdx.y * G) * p.kh * kj * kStemChannels;
  const size_t wgroup = (size_t)p.kh * kj * kStemChannels;

  float acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
  // one row of the window: an element outside the image or the slab loads the slab's first
  // element instead and is zeroed, so that no load depends on a condition
  auto row = [&](int a, auto&& each) __attribute__((always_inline)) {
    const int ih = ih0 + a;
    const bool row_ok = lane_ok && ih >= p.x_row0 && ih < p.x_row0 + p.x_rows;
    const T* const xr = xg + (size_t)(row_ok ? ih - p.x_row0 : 0) * row_elems;
    each(xr, row_ok);
  };
  auto one_row = [&](int a) __attribute__((always_inline)) {
    row(a, [&](const T* xr, bool row_ok) __attribute__((always_inline)) {
      const float* const wa = wq + (size_t)a * kj * kStemChannels;
      if constexpr (KJ != 0) {
        float xv[KJ];
#pragma unroll
        for (int j = 0; j < KJ; ++j) {
          const int e = e0 + j;
          const bool ok = row_ok && e >= 0 && e < row_elems;
          const float got = load_f32(xr + (ok ? e : 0));
          xv[j] = ok ? got : 0.f;
        }
#pragma unroll
        for (int j = 0; j < KJ; ++j)
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int c = 0; c < kStemChannels; ++c)
              acc[g * kStemChannels + c] += xv[j] * wa[g * wgroup + j * kStemChannels + c];
      } else {
        for (int j = 0; j < kj; ++j) {
          const int e = e0 + j;
          const bool ok = row_ok && e >= 0 && e < row_elems;
          const float got = load_f32(xr + (ok ? e : 0));
          const float xv = ok ? got : 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int c = 0; c < kStemChannels; ++c)
              acc[g * kStemChannels + c] += xv * wa[g * wgroup + j * kStemChannels + c];
        }
      }
    });
  };
  for (int a = 0; a < p.kh; ++a) one_row(a);   // (unrolled for 3 x 3 it measured no faster)

  // ---- bias, activation, the one rounding; CPL consecutive channels of the lane's pixel
  if (!lane_ok) return;
  const int co = blockIdx.y * CPL;
  const Clamp cl = make_clamp(p.act);
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = clamp_act(acc[c] + (p.bias ? p.bias[co + c] : 0.f), cl);
  const size_t off = ((size_t)(n * p.y_rows + oy - p.y_row0) * p.W_out + ox) * p.C_out + co;
  store_run<CPL>((T*)p.y + off, acc);
  if (p.y2) store_run<CPL>((T*)p.y2 + off, acc);
}

template <typename T, int KJ, int CPL>
__global__ __launch_bounds__(256) void conv_stem_lane_kernel(const StemParams p) {
  conv_stem_lane_kernel_body<T, KJ, CPL>(p, blockIdx.x);
}
// The same for several bands of the layer in one grid (band b owns blocks first[b] .. first[b + 1]).
template <typename T, int KJ, int CPL>
__global__ __launch_bounds__(256) void conv_stem_lane_kernel_bands(const Batch<StemParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_stem_lane_kernel_body<T, KJ, CPL>(t.p[b], blockIdx.x - t.first[b]);
}

__device__ __forceinline__ void store4(float* y, const float* v) { *(float4*)y = make_float4(v[0], v[1], v[2], v[3]); }
__device__ __forceinline__ void store4(__bf16* y, const float* v) {
  alignas(8) __bf16 o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) o[j] = (__bf16)v[j];
  *(uint2*)y = *(const uint2*)o;
}

// The form for launches too small to keep every SIMD busy with lanes that own whole pixels: a
// workgroup of four wavefronts owns 64 consecutive pixels of one output row and 16 output
// channels. It first copies the kh input rows x the columns those 64 windows touch into LDS as
// fp32 (coalesced loads along the row, zeros for padding), then lane p of wavefront w computes
// pixel p for channels 4 w .. 4 w + 3 from LDS: eight times as many wavefronts for the same
// pixels, each with an eighth of the multiply-adds.
template <typename T, int KJ>
__device__ __forceinline__ void conv_stem_kernel_body(const StemParams& p, const int bx) {
  __shared__ float patch[kStemPatchMax];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xt = bx % p.tiles_x;
  const int t = bx / p.tiles_x;
  const int r = t % p.R, n = t / p.R;
  const int oy = p.out_lo + r, ox0 = xt * kStemPixels;

  // ---- stage: kh rows x patch_w elements, element e of a row is input element iw0 * C_in + e
  const int ih0 = oy * p.sh - p.ph;
  const int e0 = (ox0 * p.sw - p.pw) * p.C_in;         // may be negative: left padding
  const int row_elems = p.W * p.C_in;
  const T* const xg = (const T*)p.x + (size_t)n * p.x_rows * row_elems;
  // (four rows at a time, every load of the batch issued before the first is used: a tap
  // outside the image or the slab loads the slab's first element instead and is zeroed after)
  for (int a0 = 0; a0 < p.kh; a0 += 4) {
    float v[4][kStemRowChunks];
#pragma unroll
    for (int da = 0; da < 4; ++da)
#pragma unroll
      for (int c = 0; c < kStemRowChunks; ++c) {
        const int ih = ih0 + a0 + da, ge = e0 + tid + c * 256;
        const bool ok = a0 + da < p.kh && tid + c * 256 < p.patch_w && ih >= p.x_row0 &&
                        ih < p.x_row0 + p.x_rows && ge >= 0 && ge < row_elems;
        const float got = load_f32(xg + (ok ? (size_t)(ih - p.x_row0) * row_elems + ge : 0));
        v[da][c] = ok ? got : 0.f;
      }
#pragma unroll
    for (int da = 0; da < 4; ++da)
#pragma unroll
      for (int c = 0; c < kStemRowChunks; ++c)
        if (a0 + da < p.kh && tid + c * 256 < p.patch_w) patch[(a0 + da) * p.patch_w + tid + c * 256] = v[da][c];
  }
  __syncthreads();

  // ---- multiply: this lane's window starts at element lane * sw * C_in of every staged row
  const int kj = KJ ? KJ : p.kw * p.C_in;               // reduction elements per kernel row
  const float* wq = p.wq + (size_t)(blockIdx.y * 4 + wave) * p.kh * kj * 4;
  const float* px = patch + lane * p.sw * p.C_in;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int a = 0; a < p.kh; ++a) {
    if constexpr (KJ != 0) {
#pragma unroll
      for (int j = 0; j < KJ; ++j) {
        const float xv = px[j];
        const float4 w4 = *(const float4*)(wq + j * 4);
        acc[0] += xv * w4.x; acc[1] += xv * w4.y; acc[2] += xv * w4.z; acc[3] += xv * w4.w;
      }
    } else {
#pragma unroll 4
      for (int j = 0; j < kj; ++j) {
        const float xv = px[j];
        const float4 w4 = *(const float4*)(wq + j * 4);
        acc[0] += xv * w4.x; acc[1] += xv * w4.y; acc[2] += xv * w4.z; acc[3] += xv * w4.w;
      }
    }
    px += p.patch_w;
    wq += kj * 4;
  }

  // ---- bias, activation, the one rounding, 4 consecutive channels per store
  const int ox = ox0 + lane;
  if (ox >= p.W_out) return;
  const int co = blockIdx.y * kStemChannels + wave * 4;
  const Clamp cl = make_clamp(p.act);
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = clamp_act(acc[j] + (p.bias ? p.bias[co + j] : 0.f), cl);
  const size_t off = ((size_t)(n * p.y_rows + oy - p.y_row0) * p.W_out + ox) * p.C_out + co;
  store4((T*)p.y + off, v);
  if (p.y2) store4((T*)p.y2 + off, v);
}

template <typename T, int KJ>
__global__ __launch_bounds__(256) void conv_stem_kernel(const StemParams p) {
  conv_stem_kernel_body<T, KJ>(p, blockIdx.x);
}
// The same for several bands of the layer in one grid (band b owns blocks first[b] .. first[b + 1]).
template <typename T, int KJ>
__global__ __launch_bounds__(256) void conv_stem_kernel_bands(const Batch<StemParams> t) {
  const int b = batch_find(t, blockIdx.x);
  conv_stem_kernel_body<T, KJ>(t.p[b], blockIdx.x - t.first[b]);
}

StemParams make_stem_params(const OpLaunch& L) {
  StemParams p;
  p.x = L.x.ptr; p.y = L.y.ptr; p.y2 = L.y2; p.wq = (const float*)L.wstem; p.bias = L.bias;
  p.wq16 = p.wq + (size_t)L.y.c * L.x.c * L.kh * L.kw;
  p.x_row0 = L.x.row0; p.x_rows = L.x.rows; p.W = L.x.w; p.C_in = L.x.c;
  p.y_row0 = L.y.row0; p.y_rows = L.y.rows; p.W_out = L.y.w; p.C_out = L.y.c;
  p.kh = L.kh; p.kw = L.kw; p.sh = L.sh; p.sw = L.sw; p.ph = L.ph; p.pw = L.pw;
  p.act = L.act; p.out_lo = L.out_lo; p.R = L.out_hi - L.out_lo; p.N = L.x.n;
  p.tiles_x = (p.W_out + kStemPixels - 1) / kStemPixels;
  p.patch_w = ((kStemPixels - 1) * p.sw + p.kw) * p.C_in;
  return p;
}

// kw * C_in if the kernel is instantiated for it (3 x 3 and 7 x 7 over 3 channels), else 0
int stem_kj(const OpLaunch& L) {
  const int kj = L.kw * L.x.c;
  return kj == 9 || kj == 21 ? kj : 0;
}

}  // namespace

bool stem_shape_applies(int c_in, int c_out, int kh, int kw, int sw, int dh, int dw, bool residual) {
  if (residual || dh != 1 || dw != 1) return false;
  if (c_in > kStemMaxCin || c_in * kh * kw > kStemMaxK || c_out % kStemChannels != 0) return false;
  const int patch_w = ((kStemPixels - 1) * sw + kw) * c_in;   // (the LDS-staged form's patch must fit)
  return patch_w <= kStemRowChunks * 256 && kh * patch_w <= kStemPatchMax;
}

bool stem_applies(const OpLaunch& L) {
  return L.op == LOP_CONV2D && L.wstem &&
         stem_shape_applies(L.x.c, L.y.c, L.kh, L.kw, L.sw, L.dh, L.dw, L.res.ptr != nullptr);
}

namespace {
// channels per lane of the lane-owned form: 32 where the layer's channels come in 32s (one pass
// over the window for twice the channels)
int stem_cpl(int c_out) { return c_out % 32 == 0 ? 32 : 16; }

// Whether a launch (all its bands together) is large enough for the lane-owned form.
bool stem_lane_pays(const StemParams* ps, int m) {
  long tiles = 0;
  for (int b = 0; b < m; ++b) tiles += (long)ps[b].N * ps[b].R * ps[b].tiles_x;
  return tiles * (ps[0].C_out / stem_cpl(ps[0].C_out)) >= kStemLaneMinWaves;
}

template <typename T, int CPL>
hipError_t launch_stem_lane(const StemParams* ps, int m, int kj, hipStream_t stream, KernelEvents* ev) {
  unsigned gx[kMaxBatch];
  for (int b = 0; b < m; ++b) gx[b] = (unsigned)(((long)ps[b].N * ps[b].R * ps[b].tiles_x + 3) / 4);   // four wavefronts, one tile each
  const unsigned gy = (unsigned)(ps[0].C_out / CPL);
  const dim3 block(256);
  if (kj == 9) return launch_group(conv_stem_lane_kernel<T, 9, CPL>, conv_stem_lane_kernel_bands<T, 9, CPL>, ps, m, gx, gy, 1, block, stream, ev);
  if (kj == 21) return launch_group(conv_stem_lane_kernel<T, 21, CPL>, conv_stem_lane_kernel_bands<T, 21, CPL>, ps, m, gx, gy, 1, block, stream, ev);
  return launch_group(conv_stem_lane_kernel<T, 0, CPL>, conv_stem_lane_kernel_bands<T, 0, CPL>, ps, m, gx, gy, 1, block, stream, ev);
}

template <typename T>
hipError_t launch_stem_staged(const StemParams* ps, int m, int kj, hipStream_t stream, KernelEvents* ev) {
  unsigned gx[kMaxBatch];
  for (int b = 0; b < m; ++b) {
    // the staged patch must fit
    if (ps[b].kh * ps[b].patch_w > kStemPatchMax || ps[b].patch_w > kStemRowChunks * 256) return hipErrorInvalidValue;
    gx[b] = (unsigned)((long)ps[b].N * ps[b].R * ps[b].tiles_x);
  }
  const unsigned gy = (unsigned)(ps[0].C_out / kStemChannels);
  const dim3 block(256);
  if (kj == 9) return launch_group(conv_stem_kernel<T, 9>, conv_stem_kernel_bands<T, 9>, ps, m, gx, gy, 1, block, stream, ev);
  if (kj == 21) return launch_group(conv_stem_kernel<T, 21>, conv_stem_kernel_bands<T, 21>, ps, m, gx, gy, 1, block, stream, ev);
  return launch_group(conv_stem_kernel<T, 0>, conv_stem_kernel_bands<T, 0>, ps, m, gx, gy, 1, block, stream, ev);
}

// Parameters of the bands of a group that compute something.
int stem_group(const OpLaunch* Ls, int n, StemParams* ps) {
  int m = 0;
  for (int b = 0; b < n && m < kMaxBatch; ++b) {
    const StemParams p = make_stem_params(Ls[b]);
    if (p.R > 0 && p.N > 0) ps[m++] = p;
  }
  return m;
}
}  // namespace

hipError_t launch_stem_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  for (int b = 0; b < n; ++b)
    if (!stem_applies(Ls[b])) return hipErrorInvalidValue;
  StemParams ps[kMaxBatch];
  const int m = stem_group(Ls, n, ps);
  if (m == 0) return hipSuccess;
  for (int b = 0; b < m; ++b) {
    if ((size_t)ps[b].x_rows * ps[b].W * ps[b].C_in == 0) return hipErrorInvalidValue;  // (padding taps load element 0)
    if ((long)ps[b].N * ps[b].R * ps[b].tiles_x > 0x7fffffffL) return hipErrorInvalidValue;
  }
  const OpLaunch& L = Ls[0];
  const int kj = stem_kj(L);
  const bool bf = L.dtype == LOP_BF16;
  if (stem_lane_pays(ps, m)) {
    if (stem_cpl(ps[0].C_out) == 32)
      return bf ? launch_stem_lane<__bf16, 32>(ps, m, kj, stream, ev) : launch_stem_lane<float, 32>(ps, m, kj, stream, ev);
    return bf ? launch_stem_lane<__bf16, 16>(ps, m, kj, stream, ev) : launch_stem_lane<float, 16>(ps, m, kj, stream, ev);
  }
  return bf ? launch_stem_staged<__bf16>(ps, m, kj, stream, ev) : launch_stem_staged<float>(ps, m, kj, stream, ev);
}

hipError_t launch_stem(const OpLaunch& L, hipStream_t stream, KernelEvents* ev) {
  return launch_stem_bands(&L, 1, stream, ev);
}

int stem_describe_bands(const OpLaunch* Ls, int n, char* name, size_t size) {
  const OpLaunch& L = Ls[0];
  StemParams ps[kMaxBatch];
  const int m = n >= 1 && n <= kMaxBatch ? stem_group(Ls, n, ps) : 0;
  const char* const form = m > 1 ? "_bands" : "";
  const char* const type = L.dtype == LOP_BF16 ? "__bf16" : "float";
  if (name && size) {
    if (m > 0 && stem_lane_pays(ps, m))
      snprintf(name, size, "conv_stem_lane_kernel%s<%s, %d, %d>", form, type, stem_kj(L), stem_cpl(L.y.c));
    else
      snprintf(name, size, "conv_stem_kernel%s<%s, %d>", form, type, stem_kj(L));
  }
  return 1;
}

int stem_describe(const OpLaunch& L, char* name, size_t size) { return stem_describe_bands(&L, 1, name, size); }

}  // namespace lop
