// Bandwidth-bound local operators on a row interval: depthwise convolution, max pooling
// and the stand-alone element-wise operator (Intra-DP Sec. IV-A: block-wise and
// element-wise local operators). NHWC: a thread owns one 16-byte channel vector of one
// output pixel, consecutive threads own consecutive channel vectors, so every load and
// store of a wavefront is one contiguous run of channels. fp32 math, one rounding.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "act.hpp"
#include "kernels.hpp"
#include "launch.hpp"
#include "lop.h"

namespace lop {
namespace {

struct RowParams {
  const void* x;
  void* y;
  void* y2;  // second destination with y's layout, or nullptr
  const void* res;
  const float* w;  // depthwise: [kh*kw][C] fp32
  const float* bias;
  int x_row0, x_rows, W, C;
  int y_row0, y_rows, W_out;
  int r_row0, r_rows;
  int kh, kw, sh, sw, ph, pw, dh, dw;
  int act, out_lo, R, N;
  long total;  // N * R * W_out * (C / VEC)
};

template <typename T, int VEC> struct Vec;  // VEC elements of T <-> fp32 registers

template <> struct Vec<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float* v) {
    const float4 t = *(const float4*)p; v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float* v) { v[0] = *p; }
  static __device__ __forceinline__ void store(float* p, const float* v) { *p = v[0]; }
};
template <> struct Vec<__bf16, 8> {
  static __device__ __forceinline__ void load(const __bf16* p, float* v) {
    const uint4 t = *(const uint4*)p;
    const unsigned u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(u[i] << 16);
      v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(__bf16* p, const float* v) {
    alignas(16) __bf16 o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (__bf16)v[i];
    *(uint4*)p = *(const uint4*)o;
  }
};
template <> struct Vec<__bf16, 4> {
  static __device__ __forceinline__ void load(const __bf16* p, float* v) {
    const uint2 t = *(const uint2*)p;
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(__bf16* p, const float* v) {
    alignas(8) __bf16 o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (__bf16)v[i];
    *(uint2*)p = *(const uint2*)o;
  }
};
template <> struct Vec<__bf16, 1> {
  static __device__ __forceinline__ void load(const __bf16* p, float* v) { v[0] = (float)*p; }
  static __device__ __forceinline__ void store(__bf16* p, const float* v) { *p = (__bf16)v[0]; }
};

template <int VEC>
__device__ __forceinline__ void load_f32(const float* p, float* v) {
  if constexpr (VEC >= 4) {
#pragma unroll
    for (int i = 0; i < VEC; i += 4) {
      const float4 t = *(const float4*)(p + i);
      v[i] = t.x; v[i + 1] = t.y; v[i + 2] = t.z; v[i + 3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = p[i];
  }
}

// OP: 0 depthwise conv, 1 max pool, 2 element-wise
template <typename T, int VEC, int OP>
__device__ __forceinline__ void rowwise_kernel_body(const RowParams& p, const int bx) {
  const long gid = (long)bx * 256 + threadIdx.x;
  if (gid >= p.total) return;
  const int cv = p.C / VEC;
  const int c = (int)(gid % cv) * VEC;
  long t = gid / cv;
  const int ow = (int)(t % p.W_out);
  t /= p.W_out;
  const int r = (int)(t % p.R), n = (int)(t / p.R);
  const int oh = p.out_lo + r;
  const T* __restrict__ xg = (const T*)p.x;
  float acc[VEC];
  if (OP == 2) {
    Vec<T, VEC>::load(xg + ((size_t)(n * p.x_rows + oh - p.x_row0) * p.W + ow) * p.C + c, acc);
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = OP == 1 ? -INFINITY : 0.f;
    const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
    for (int a = 0; a < p.kh; ++a) {
      const int ih = ih0 + a * p.dh;
      if (ih < p.x_row0 || ih >= p.x_row0 + p.x_rows) continue;
      for (int b = 0; b < p.kw; ++b) {
        const int iw = iw0 + b * p.dw;
        if (iw < 0 || iw >= p.W) continue;
        float v[VEC];
        Vec<T, VEC>::load(xg + ((size_t)(n * p.x_rows + ih - p.x_row0) * p.W + iw) * p.C + c, v);
        if (OP == 1) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = fmaxf(acc[i], v[i]);
        } else {
          float wv[VEC];
          load_f32<VEC>(p.w + (size_t)(a * p.kw + b) * p.C + c, wv);
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] = fmaf(v[i], wv[i], acc[i]);
        }
      }
    }
  }
  if (OP != 1) {
    if (p.bias) {
      float bv[VEC];
      load_f32<VEC>(p.bias + c, bv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += bv[i];
    }
    if (p.res) {
      float rv[VEC];
      Vec<T, VEC>::load((const T*)p.res +
                            ((size_t)(n * p.r_rows + oh - p.r_row0) * p.W_out + ow) * p.C + c, rv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += rv[i];
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = clamp_act(acc[i], make_clamp(p.act));
  }
  const size_t yo = ((size_t)(n * p.y_rows + oh - p.y_row0) * p.W_out + ow) * p.C + c;
  Vec<T, VEC>::store((T*)p.y + yo, acc);
  if (p.y2) Vec<T, VEC>::store((T*)p.y2 + yo, acc);
}

template <typename T, int VEC, int OP>
__global__ __launch_bounds__(256) void rowwise_kernel(const RowParams p) {
  rowwise_kernel_body<T, VEC, OP>(p, blockIdx.x);
}
// The same for several bands of one layer in one grid (band b owns blocks first[b] .. first[b + 1]).
template <typename T, int VEC, int OP>
__global__ __launch_bounds__(256) void rowwise_kernel_bands(const Batch<RowParams> t) {
  const int b = batch_find(t, blockIdx.x);
  rowwise_kernel_body<T, VEC, OP>(t.p[b], blockIdx.x - t.first[b]);
}


// Depthwise 3x3 (dilation 1, pad 1, stride S in both directions), register blocked: a
// thread owns VEC channels of one output column and dw_rows_per_thread(S) consecutive output
// rows; it loads the (rows-1)*S + 3 input rows it needs (3 vectors each) and the 9 x VEC
// weights once, so an output costs about S + 0.5 vector loads instead of 9 loads plus 9
// weight loads. Threads of a workgroup are (channel vector, column) with the channel
// vector fastest: loads and stores of a wavefront stay contiguous and the left/right
// neighbours' columns come out of the same CU's L1. No residual (rowwise_kernel has it).
// Output rows per thread: the (rows - 1) * S + 3 input rows are read once per thread, so the
// rows shared with the chunk above and below are fetched twice: 6 for 4 with stride 1 (1.5 x),
// 10 for 8 (1.25 x); with stride 2, 9 for 4 is 1.125 x already.
constexpr int dw_rows_per_thread(int stride) { return stride == 1 ? 8 : 4; }
struct Dw3Params {
  RowParams r;
  int cols_per_block;  // output columns per workgroup
  int chunks;          // row chunks (dw_rows_per_thread output rows each) per image
};

// Raw 8- or 16-byte vector of the storage type and its expansion to fp32 values.
template <int BYTES> struct RawVec;
template <> struct RawVec<16> { typedef uint4 type; };
template <> struct RawVec<8> { typedef uint2 type; };

__device__ __forceinline__ void unpack_bf16(const uint4& t, float* v) {
  const unsigned u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(u[i] << 16);
    v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void unpack_bf16(const uint2& t, float* v) {
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}
__device__ __forceinline__ void unpack_f32(const uint4& t, float* v) {
  v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y);
  v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
}
template <typename T, typename R>
__device__ __forceinline__ void unpack(const R& t, float* v) {
  if constexpr (sizeof(T) == 2) unpack_bf16(t, v);
  else unpack_f32(t, v);
}

template <typename T, int VEC, int S>
__global__ __launch_bounds__(256) void dwconv3x3_kernel(const Dw3Params q) {
  static_assert(VEC * sizeof(T) == 16 || VEC * sizeof(T) == 8, "8- or 16-byte vectors");
  typedef typename RawVec<VEC * sizeof(T)>::type Raw;
  constexpr int RPT = dw_rows_per_thread(S);  // output rows per thread
  constexpr int NR = (RPT - 1) * S + 3;    // input rows they read
  const RowParams& p = q.r;
  const int cv = p.C / VEC;
  const int cg = threadIdx.x % cv, col = threadIdx.x / cv;
  const int ow = blockIdx.x * q.cols_per_block + col;
  if (col >= q.cols_per_block || ow >= p.W_out) return;
  const int chunk = blockIdx.y % q.chunks, n = blockIdx.y / q.chunks;
  const int c = cg * VEC;
  const int oh0 = p.out_lo + chunk * RPT;
  const int oh1 = min(oh0 + RPT, p.out_lo + p.R);
  const T* __restrict__ xg = (const T*)p.x;
  T* __restrict__ yg = (T*)p.y;
  const Clamp clamp = make_clamp(p.act);

  // Every load first (input rows, weights, bias), all stores after: loads and stores share
  // one in-order counter, so a load waited for after a store would wait for the store too.
  Raw in[NR][3];
  const int ih0 = oh0 * S - 1, iw0 = ow * S - 1;
  const int rows_needed = (oh1 - oh0 - 1) * S + 3;
#pragma unroll
  for (int a = 0; a < NR; ++a) {
    const int ih = ih0 + a;
    const bool row_ok = a < rows_needed && ih >= p.x_row0 && ih < p.x_row0 + p.x_rows;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      const int iw = iw0 + b;
      in[a][b] = Raw{};
      if (row_ok && iw >= 0 && iw < p.W)
        in[a][b] = *(const Raw*)(xg + ((size_t)(n * p.x_rows + ih - p.x_row0) * p.W + iw) * p.C + c);
    }
  }
  float w[9][VEC];
#pragma unroll
  for (int t = 0; t < 9; ++t) load_f32<VEC>(p.w + (size_t)t * p.C + c, w[t]);
  float bias[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) bias[i] = 0.f;
  if (p.bias) load_f32<VEC>(p.bias + c, bias);

#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    if (oh0 + r >= oh1) break;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = bias[i];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
      for (int b = 0; b < 3; ++b) {
        float x[VEC];
        unpack<T>(in[r * S + a][b], x);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = fmaf(x[i], w[a * 3 + b][i], acc[i]);
      }
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = clamp_act(acc[i], clamp);
    const size_t yo = ((size_t)(n * p.y_rows + oh0 + r - p.y_row0) * p.W_out + ow) * p.C + c;
    Vec<T, VEC>::store(yg + yo, acc);
    if (p.y2) Vec<T, VEC>::store((T*)p.y2 + yo, acc);
  }
}

// The sliding-window kernel covers the common depthwise case; everything else runs on
// rowwise_kernel.
inline bool dw3_applies(const RowParams& p, int op, int vec) {
  return op == LOP_DWCONV2D && p.kh == 3 && p.kw == 3 && p.dh == 1 && p.dw == 1 && p.ph == 1 &&
         p.pw == 1 && p.sh == p.sw && (p.sh == 1 || p.sh == 2) && vec > 1 && p.C / vec <= 256 &&
         p.res == nullptr;
}

template <typename T, int VEC>
hipError_t launch_dw3(const RowParams& p, hipStream_t s, KernelEvents* ev) {
  if (p.R <= 0) return hipSuccess;
  Dw3Params q;
  q.r = p;
  const int cv = p.C / VEC;
  q.cols_per_block = std::max(1, 256 / cv);
  const int rpt = dw_rows_per_thread(p.sh);
  q.chunks = (p.R + rpt - 1) / rpt;
  dim3 grid((p.W_out + q.cols_per_block - 1) / q.cols_per_block, q.chunks * p.N);
  return p.sh == 1 ? launch_kernel(dwconv3x3_kernel<T, VEC, 1>, grid, dim3(256), s, ev, q)
                   : launch_kernel(dwconv3x3_kernel<T, VEC, 2>, grid, dim3(256), s, ev, q);
}

// Channel vector per thread of the sliding-window kernel (0: it does not apply).
inline int dw3_vec(const RowParams& p, int op, int dtype) {
  (void)dtype;
  const int want = 4;
  if (p.C % want != 0) return 0;
  return dw3_applies(p, op, want) ? want : 0;
}

template <typename T, int VEC>
hipError_t launch_rowwise(RowParams* ps, int n, int op, hipStream_t s, KernelEvents* ev) {
  unsigned gx[kMaxBatch];
  int m = 0;
  for (int b = 0; b < n; ++b) {
    ps[b].total = (long)ps[b].N * ps[b].R * ps[b].W_out * (ps[b].C / VEC);
    if (ps[b].total <= 0) continue;
    ps[m] = ps[b];
    gx[m++] = (unsigned)((ps[b].total + 255) / 256);
  }
  if (m == 0) return hipSuccess;
  if (op == LOP_DWCONV2D)
    return launch_group(rowwise_kernel<T, VEC, 0>, rowwise_kernel_bands<T, VEC, 0>, ps, m, gx, 1, 1, dim3(256), s, ev);
  if (op == LOP_MAXPOOL2D)
    return launch_group(rowwise_kernel<T, VEC, 1>, rowwise_kernel_bands<T, VEC, 1>, ps, m, gx, 1, 1, dim3(256), s, ev);
  return launch_group(rowwise_kernel<T, VEC, 2>, rowwise_kernel_bands<T, VEC, 2>, ps, m, gx, 1, 1, dim3(256), s, ev);
}

RowParams make_row_params(const OpLaunch& L) {
  RowParams p;
  p.x = L.x.ptr; p.y = L.y.ptr; p.y2 = L.y2; p.res = L.res.ptr; p.w = (const float*)L.w; p.bias = L.bias;
  p.x_row0 = L.x.row0; p.x_rows = L.x.rows; p.W = L.x.w; p.C = L.x.c;
  p.y_row0 = L.y.row0; p.y_rows = L.y.rows; p.W_out = L.y.w;
  p.r_row0 = L.res.row0; p.r_rows = L.res.rows;
  p.kh = L.kh; p.kw = L.kw; p.sh = L.sh; p.sw = L.sw; p.ph = L.ph; p.pw = L.pw;
  p.dh = L.dh; p.dw = L.dw;
  p.act = L.act; p.out_lo = L.out_lo; p.R = L.out_hi - L.out_lo; p.N = L.x.n;
  p.total = 0;
  return p;
}

}  // namespace

// Whether launch_rowwise_bands has a kernel for this operator (the register-blocked depthwise
// kernel takes one band at a time).
bool rowwise_batchable(const OpLaunch& L) {
  const RowParams p = make_row_params(L);
  return dw3_vec(p, L.op, L.dtype) == 0;
}

hipError_t launch_rowwise_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev) {
  if (n < 1 || n > kMaxBatch) return hipErrorInvalidValue;
  RowParams ps[kMaxBatch];
  for (int b = 0; b < n; ++b) ps[b] = make_row_params(Ls[b]);
  const OpLaunch& L = Ls[0];
  RowParams& p = ps[0];
  if (const int v = dw3_vec(p, L.op, L.dtype)) {
    if (n != 1) return hipErrorInvalidValue;
    if (L.dtype != LOP_BF16) return launch_dw3<float, 4>(p, stream, ev);
    return v == 8 ? launch_dw3<__bf16, 8>(p, stream, ev) : launch_dw3<__bf16, 4>(p, stream, ev);
  }
  if (L.dtype == LOP_BF16)
    return p.C % 8 == 0 ? launch_rowwise<__bf16, 8>(ps, n, L.op, stream, ev)
                        : launch_rowwise<__bf16, 1>(ps, n, L.op, stream, ev);
  return p.C % 4 == 0 ? launch_rowwise<float, 4>(ps, n, L.op, stream, ev)
                      : launch_rowwise<float, 1>(ps, n, L.op, stream, ev);
}

hipError_t launch_rowwise_op(const OpLaunch& L, hipStream_t stream, KernelEvents* ev) {
  return launch_rowwise_bands(&L, 1, stream, ev);
}

namespace {
// Copies `n` segments of `len` bytes (segment i at offset i*pitch in both buffers), 16 bytes
// per thread and step. Used to push a band's finished rows into mapped pinned host memory
// from a stream of its own: the stores travel over PCIe while other streams compute.
__global__ __launch_bounds__(256) void copy_rows_kernel(char* __restrict__ dst,
                                                        const char* __restrict__ src,
                                                        size_t pitch, size_t len, int n) {
  const size_t vec = len / 16;
  const size_t stride = (size_t)gridDim.x * 256;
  for (int i = 0; i < n; ++i) {
    const uint4* s = (const uint4*)(src + i * pitch);
    uint4* d = (uint4*)(dst + i * pitch);
    for (size_t j = (size_t)blockIdx.x * 256 + threadIdx.x; j < vec; j += stride) d[j] = s[j];
    // tail bytes (len is a multiple of the element size, not necessarily of 16)
    for (size_t j = vec * 16 + (size_t)blockIdx.x * 256 + threadIdx.x; j < len; j += stride)
      dst[i * pitch + j] = src[i * pitch + j];
  }
}
// Fills `bytes` (a multiple of 16) with one 32-bit pattern: the debug poisoning of scratch
// memory (a kernel, not a memset, so that it may be captured into a graph).
__global__ __launch_bounds__(256) void fill_words_kernel(uint4* __restrict__ dst, size_t vecs, unsigned word) {
  const size_t stride = (size_t)gridDim.x * 256;
  const uint4 v = make_uint4(word, word, word, word);
  for (size_t j = (size_t)blockIdx.x * 256 + threadIdx.x; j < vecs; j += stride) dst[j] = v;
}
}  // namespace

hipError_t launch_fill_words(void* dst, size_t bytes, unsigned word, hipStream_t stream) {
  const size_t vecs = bytes / 16;
  if (!dst || vecs == 0) return hipSuccess;
  const unsigned grid = (unsigned)std::min<size_t>((vecs + 255) / 256, 2048);
  hipLaunchKernelGGL(fill_words_kernel, dim3(grid), dim3(256), 0, stream, (uint4*)dst, vecs, word);
  return hipGetLastError();
}

hipError_t launch_copy_rows(void* dst, const void* src, size_t pitch, size_t len, int n,
                            hipStream_t stream, int workgroups) {
  if (len == 0 || n <= 0) return hipSuccess;
  const size_t vec = (len + 15) / 16;
  // Few workgroups on purpose: the stores are paced by PCIe, and many of them in flight
  // hold up the HBM writes of the kernels running beside the copy (4 workgroups still move
  // about 30 GB/s; with 64 the copy was 1.7x faster and the other streams lost more than that).
  const unsigned grid = (unsigned)std::min<size_t>((vec + 255) / 256, (size_t)std::max(1, workgroups));
  hipLaunchKernelGGL(copy_rows_kernel, dim3(grid), dim3(256), 0, stream, (char*)dst,
                     (const char*)src, pitch, len, n);
  return hipGetLastError();
}

int rowwise_describe(const OpLaunch& L, char* name, size_t size) {
  const bool bf = L.dtype == LOP_BF16;
  const int vec = bf ? (L.x.c % 8 == 0 ? 8 : 1) : (L.x.c % 4 == 0 ? 4 : 1);
  const int o = L.op == LOP_DWCONV2D ? 0 : (L.op == LOP_MAXPOOL2D ? 1 : 2);
  RowParams p;
  p.kh = L.kh; p.kw = L.kw; p.sh = L.sh; p.sw = L.sw; p.ph = L.ph; p.pw = L.pw;
  p.dh = L.dh; p.dw = L.dw; p.C = L.x.c; p.res = L.res.ptr;
  if (name && size) {
    if (const int v = dw3_vec(p, L.op, L.dtype))
      snprintf(name, size, "dwconv3x3_kernel<%s, %d, %d>", bf ? "__bf16" : "float", v, L.sh);
    else
      snprintf(name, size, "rowwise_kernel<%s, %d, %d>", bf ? "__bf16" : "float", vec, o);
  }
  return 1;
}

}  // namespace lop
