// Inverted-residual block in one launch: 1x1 expand + activation, depthwise 3x3 (stride 1 or 2)
// + activation, 1x1 project (+ residual), on a row interval of the block's output.
//
// The three operators are local (Intra-DP Sec. IV-A: a block-wise operator between two
// row-wise ones, Eq. 1), so a tile of the block's output depends on a slightly larger tile of
// its input only. Run layer by layer the expanded tensor (6x the channels) is written to HBM
// and read back twice; here it never leaves the compute unit. A workgroup owns a TH x TW tile
// of output pixels and walks over the expanded channels in chunks of 32:
//   expand   MFMA: the chunk's 32 channels for the (TH-1)S+3 x (TW-1)S+3 input pixels the
//            tile's depthwise windows touch -> bias, activation, one rounding to bf16 -> LDS.
//            Pixels outside the image are zero there (the depthwise operator pads its input,
//            i.e. the expanded tensor, not the block's input);
//   depthwise  also on MFMA, as nine products with diagonal weight matrices (one per tap)
//            whose other operand is the expanded tile shifted by the tap: 31/32 of those
//            multiplications are by zero, but the matrix pipe has them to spare, reads bf16
//            directly and accumulates in fp32, while the same arithmetic on the vector ALUs
//            (unpack, 9 FMAs per value) was the kernel's bottleneck -> bias, activation, one
//            rounding -> LDS;
//   project  MFMA: adds the chunk's contribution to the 32 output channels (accumulators stay
//            in registers over the chunks).
// The roundings are the ones the layer-by-layer path makes, so results agree with it to fp32
// summation order. Shapes: 32 input and 32 output channels, up to 192 expanded channels, bf16.
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
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMbC = 32;          // input and output channels
constexpr int kMbMaxMid = 192;    // expanded channels held by the staged depthwise weights

struct MbParams {
  const __bf16* x;
  __bf16* y;
  const __bf16* res;
  const __bf16* we;   // expand weights [c_mid padded][ke_pad]
  const float* be;
  const float* wd;    // depthwise weights [tap][C_mid]
  const float* bd;
  const __bf16* wp;   // project weights [32 padded][kp_pad]
  const float* bp;
  int ke_pad, kp_pad;
  int x_row0, x_rows, H, W;
  int y_row0, y_rows, W_out;
  int r_row0, r_rows;
  int C_mid, nch;
  Clamp ce, cd, cp;
  int out_lo, R, N;
  int tiles_x, tiles_y;
};

__device__ __forceinline__ f32x16 mma_bf16(const u32x4& a, const u32x4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// four bf16 (8 bytes) <-> four floats
__device__ __forceinline__ void unpack4(const u32x2& v, float* f) {
  f[0] = __builtin_bit_cast(float, v.x << 16);
  f[1] = __builtin_bit_cast(float, v.x & 0xffff0000u);
  f[2] = __builtin_bit_cast(float, v.y << 16);
  f[3] = __builtin_bit_cast(float, v.y & 0xffff0000u);
}
__device__ __forceinline__ u32x2 pack4(const float* f) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 b;
  b[0] = (__bf16)f[0]; b[1] = (__bf16)f[1]; b[2] = (__bf16)f[2]; b[3] = (__bf16)f[3];
  return __builtin_bit_cast(u32x2, b);
}

template <int S>
struct MbTile {
  static constexpr int TH = 8, TW = 16;                  // output pixels of a workgroup
  static constexpr int EH = (TH - 1) * S + 3, EW = (TW - 1) * S + 3;  // expanded pixels it needs
  static constexpr int EP = EH * EW;
  static constexpr int MT_E = (EP + 31) / 32;            // expand MFMA tiles
  static constexpr int MPW = (MT_E + 3) / 4;             // ... per wavefront
  static constexpr int OP = TH * TW;                     // = 4 MFMA tiles, one per wavefront
  static constexpr int PITCH = 80;                       // bytes per pixel in LDS (64 + pad)
};

template <int S, bool RES>
__global__ __launch_bounds__(256, S == 1 ? 4 : 2) void mbconv_kernel(const MbParams p) {
  typedef MbTile<S> G;
  constexpr int TH = G::TH, TW = G::TW, EW = G::EW, EP = G::EP, MT_E = G::MT_E, MPW = G::MPW;
  constexpr int EPITCH = G::PITCH, DPITCH = G::PITCH;
  static_assert(G::OP == 128, "one 32-pixel MFMA tile of the output per wavefront");
  __shared__ __attribute__((aligned(16))) unsigned char E_s[MT_E * 32 * EPITCH];
  __shared__ __attribute__((aligned(16))) unsigned char D_s[G::OP * DPITCH];
  __shared__ __attribute__((aligned(16))) float wd_s[10 * kMbMaxMid];  // 9 taps, then the bias
  __shared__ __attribute__((aligned(16))) float be_s[kMbMaxMid];       // expand bias

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int px = lane & 31, kg = lane >> 5;
  int bid = blockIdx.x;
  const int tx = bid % p.tiles_x;
  bid /= p.tiles_x;
  const int ty = bid % p.tiles_y;
  const int n = bid / p.tiles_y;
  const int oh0 = p.out_lo + ty * TH, ow0 = tx * TW;
  const int ih_base = oh0 * S - 1, iw_base = ow0 * S - 1;

  // stage the depthwise weights and the two biases: all loads first (a loop of load-store
  // pairs would pay the memory latency once per trip)
  {
    const int nw4 = 9 * p.C_mid / 4, nb4 = p.C_mid / 4;  // float4 counts (<= 432, <= 48)
    float4 w0 = make_float4(0.f, 0.f, 0.f, 0.f), w1 = w0, b0 = w0, b1 = w0;
    if (tid < nw4) w0 = ((const float4*)p.wd)[tid];
    if (tid + 256 < nw4) w1 = ((const float4*)p.wd)[tid + 256];
    if (tid < nb4 && p.bd) b0 = ((const float4*)p.bd)[tid];
    if (tid < nb4 && p.be) b1 = ((const float4*)p.be)[tid];
    if (tid < nw4) ((float4*)wd_s)[tid] = w0;
    if (tid + 256 < nw4) ((float4*)wd_s)[tid + 256] = w1;
    if (tid < nb4) {
      ((float4*)(wd_s + 9 * p.C_mid))[tid] = b0;
      ((float4*)be_s)[tid] = b1;
    }
  }

  // ---- the block's input at the expanded pixels of this wavefront's MFMA tiles, in operand
  // layout (lane = pixel, two halves of 8 channels per step of 16), kept for all chunks
  u32x4 xa[MPW][2];
  bool xin[MPW];
#pragma unroll
  for (int i = 0; i < MPW; ++i) {
    const int e = (wave + 4 * i) * 32 + px;
    const int er = e / EW, ec = e - er * EW;
    const int ih = ih_base + er, iw = iw_base + ec;
    xin[i] = wave + 4 * i < MT_E && e < EP && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W &&
             ih >= p.x_row0 && ih < p.x_row0 + p.x_rows;
    xa[i][0] = u32x4{0u, 0u, 0u, 0u};
    xa[i][1] = u32x4{0u, 0u, 0u, 0u};
    if (xin[i]) {
      const __bf16* src = p.x + ((size_t)(n * p.x_rows + ih - p.x_row0) * p.W + iw) * kMbC + kg * 8;
      xa[i][0] = *(const u32x4*)src;
      xa[i][1] = *(const u32x4*)(src + 16);
    }
  }

  // this lane's output pixel (of the wavefront's 32) and where its window starts in E_s
  const int o = wave * 32 + px;
  const int orow = o / TW, ocol = o - orow * TW;
  const unsigned char* const ewin = E_s + ((orow * S) * EW + ocol * S) * EPITCH + kg * 16;
  // diagonal weight matrices as MFMA A operands: row (= channel) chl has its one non-zero at
  // k = chl, i.e. in step chl / 16, lane half (chl % 16) / 8, slot chl % 8 of the 8 bf16
  const int chl = lane & 31;
  unsigned amask[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      amask[j][i] = ((chl >> 4) == j && ((chl >> 3) & 1) == kg && ((chl & 7) >> 1) == i) ? 0xffffffffu : 0u;
  const int wshift = (chl & 1) * 16;

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  // weight fragments (MFMA A operands) of a chunk: expand rows c*32 + px, project columns
  // c*32 ...; the next chunk's are fetched while this one is worked on
  u32x4 wef[2], wpf[2];
  auto fetch_weights = [&](int c, u32x4 (&we2)[2], u32x4 (&wp2)[2]) __attribute__((always_inline)) {
    const __bf16* wr = p.we + (size_t)(c * 32 + px) * p.ke_pad + kg * 8;
    we2[0] = *(const u32x4*)wr;
    we2[1] = *(const u32x4*)(wr + 16);
    const __bf16* pr = p.wp + (size_t)px * p.kp_pad + c * 32 + kg * 8;
    wp2[0] = *(const u32x4*)pr;
    wp2[1] = *(const u32x4*)(pr + 16);
  };
  fetch_weights(0, wef, wpf);
  __syncthreads();  // staged biases and depthwise weights are in LDS

  for (int c = 0; c < p.nch; ++c) {
    u32x4 wef_n[2] = {wef[0], wef[1]}, wpf_n[2] = {wpf[0], wpf[1]};
    if (c + 1 < p.nch) fetch_weights(c + 1, wef_n, wpf_n);
    float4 eb[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) eb[g] = *(const float4*)(be_s + c * 32 + g * 8 + kg * 4);

    // ---- expand: lane ends with channels g*8 + kg*4 + {0..3} of pixel px
#pragma unroll
    for (int i = 0; i < MPW; ++i) {
      const int mt = wave + 4 * i;
      if (mt >= MT_E) continue;
      f32x16 a;
#pragma unroll
      for (int k = 0; k < 16; ++k) a[k] = 0.f;
      a = mma_bf16(wef[0], xa[i][0], a);
      a = mma_bf16(wef[1], xa[i][1], a);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v[4];
        v[0] = clamp_act(a[g * 4 + 0] + eb[g].x, p.ce);
        v[1] = clamp_act(a[g * 4 + 1] + eb[g].y, p.ce);
        v[2] = clamp_act(a[g * 4 + 2] + eb[g].z, p.ce);
        v[3] = clamp_act(a[g * 4 + 3] + eb[g].w, p.ce);
        u32x2 pk = pack4(v);
        if (!xin[i]) pk = u32x2{0u, 0u};  // padding of the depthwise operator
        *(u32x2*)(E_s + (mt * 32 + px) * EPITCH + g * 16 + kg * 8) = pk;
      }
    }
    __syncthreads();

    // ---- depthwise 3x3 on the chunk: D[ch][px] = sum over taps of diag(w_tap) x E(px + tap)
    {
      f32x16 d0, d1;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b4 = *(const float4*)(wd_s + 9 * p.C_mid + c * 32 + g * 8 + kg * 4);
        d0[g * 4 + 0] = b4.x; d0[g * 4 + 1] = b4.y; d0[g * 4 + 2] = b4.z; d0[g * 4 + 3] = b4.w;
      }
#pragma unroll
      for (int k = 0; k < 16; ++k) d1[k] = 0.f;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        // the weights are bf16 values held as fp32: the upper 16 bits are the value
        const unsigned wv = (__builtin_bit_cast(unsigned, wd_s[t * p.C_mid + c * 32 + chl]) >> 16) << wshift;
        const u32x4 a0 = u32x4{wv & amask[0][0], wv & amask[0][1], wv & amask[0][2], wv & amask[0][3]};
        const u32x4 a1 = u32x4{wv & amask[1][0], wv & amask[1][1], wv & amask[1][2], wv & amask[1][3]};
        const unsigned char* src = ewin + ((t / 3) * EW + (t % 3)) * EPITCH;
        d0 = mma_bf16(a0, *(const u32x4*)src, d0);
        d1 = mma_bf16(a1, *(const u32x4*)(src + 32), d1);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = clamp_act(d0[g * 4 + k] + d1[g * 4 + k], p.cd);
        *(u32x2*)(D_s + o * DPITCH + g * 16 + kg * 8) = pack4(v);
      }
    }
    __syncthreads();

    // ---- project: this chunk's 32 channels are the reduction axis
    {
      const unsigned char* src = D_s + o * DPITCH + kg * 16;
      const u32x4 b0 = *(const u32x4*)src;
      const u32x4 b1 = *(const u32x4*)(src + 32);
      acc = mma_bf16(wpf[0], b0, acc);
      acc = mma_bf16(wpf[1], b1, acc);
    }
    wef[0] = wef_n[0]; wef[1] = wef_n[1];
    wpf[0] = wpf_n[0]; wpf[1] = wpf_n[1];
  }

  // ---- bias, residual, activation, the one rounding; 8 bytes per lane and channel group
  const int oh = oh0 + orow, ow = ow0 + ocol;
  if (oh >= p.out_lo + p.R || ow >= p.W_out) return;
  const size_t yoff = ((size_t)(n * p.y_rows + oh - p.y_row0) * p.W_out + ow) * kMbC;
  const size_t roff = RES ? ((size_t)(n * p.r_rows + oh - p.r_row0) * p.W_out + ow) * kMbC : 0;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int co = g * 8 + kg * 4;
    float v[4] = {acc[g * 4 + 0], acc[g * 4 + 1], acc[g * 4 + 2], acc[g * 4 + 3]};
    if (p.bp) {
      const float4 b4 = *(const float4*)(p.bp + co);
      v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
    }
    if (RES) {
      float r[4];
      unpack4(*(const u32x2*)(p.res + roff + co), r);
      v[0] += r[0]; v[1] += r[1]; v[2] += r[2]; v[3] += r[3];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = clamp_act(v[k], p.cp);
    *(u32x2*)(p.y + yoff + co) = pack4(v);
  }
}

bool is_pointwise(const OpLaunch& L) {
  return L.op == LOP_CONV2D && L.kh == 1 && L.kw == 1 && L.sh == 1 && L.sw == 1 && L.ph == 0 &&
         L.pw == 0;
}

}  // namespace

// Whether the three operators (expand, depthwise, project; shapes and parameters only, the
// slabs are not looked at) can run as one mbconv_kernel launch.
bool mbconv_applies(const OpLaunch& e, const OpLaunch& d, const OpLaunch& p) {
  if (e.dtype != LOP_BF16 || !is_pointwise(e) || !is_pointwise(p)) return false;
  if (e.x.c != kMbC || p.y.c != kMbC) return false;
  if (e.y.c % 32 != 0 || e.y.c > kMbMaxMid || e.y.c != d.x.c || d.x.c != p.x.c) return false;
  if (d.op != LOP_DWCONV2D || d.kh != 3 || d.kw != 3 || d.ph != 1 || d.pw != 1 || d.dh != 1 ||
      d.dw != 1 || d.sh != d.sw || (d.sh != 1 && d.sh != 2))
    return false;
  return e.res.ptr == nullptr && d.res.ptr == nullptr;
}

int mbconv_describe(const OpLaunch& d, const OpLaunch& p, char* name, size_t size) {
  if (name && size)
    snprintf(name, size, "mbconv_kernel<%d, %s>", d.sh, p.res.ptr ? "true" : "false");
  return 1;
}

// e.x: the block's input slab; p.y: its output slab; p.res: residual slab or none;
// p.out_lo/out_hi: the output rows to produce.
hipError_t launch_mbconv(const OpLaunch& e, const OpLaunch& d, const OpLaunch& p, hipStream_t stream,
                         KernelEvents* ev) {
  if (!mbconv_applies(e, d, p)) return hipErrorInvalidValue;
  MbParams q;
  q.x = (const __bf16*)e.x.ptr; q.y = (__bf16*)p.y.ptr; q.res = (const __bf16*)p.res.ptr;
  q.we = (const __bf16*)e.w; q.be = e.bias;
  q.wd = (const float*)d.w; q.bd = d.bias;
  q.wp = (const __bf16*)p.w; q.bp = p.bias;
  q.ke_pad = e.k_pad; q.kp_pad = p.k_pad;
  q.x_row0 = e.x.row0; q.x_rows = e.x.rows; q.H = e.x.h; q.W = e.x.w;
  q.y_row0 = p.y.row0; q.y_rows = p.y.rows; q.W_out = p.y.w;
  q.r_row0 = p.res.row0; q.r_rows = p.res.rows;
  q.C_mid = e.y.c; q.nch = e.y.c / 32;
  q.ce = make_clamp(e.act); q.cd = make_clamp(d.act); q.cp = make_clamp(p.act);
  q.out_lo = p.out_lo; q.R = p.out_hi - p.out_lo; q.N = e.x.n;
  if (q.R <= 0 || q.N <= 0) return hipSuccess;
  const int s = d.sh;
  const int tw = MbTile<1>::TW, th = MbTile<1>::TH;
  q.tiles_x = (q.W_out + tw - 1) / tw;
  q.tiles_y = (q.R + th - 1) / th;
  const dim3 grid((unsigned)(q.tiles_x * q.tiles_y * q.N));
  if (s == 1)
    return q.res ? launch_kernel(mbconv_kernel<1, true>, grid, dim3(256), stream, ev, q)
                 : launch_kernel(mbconv_kernel<1, false>, grid, dim3(256), stream, ev, q);
  return q.res ? launch_kernel(mbconv_kernel<2, true>, grid, dim3(256), stream, ev, q)
               : launch_kernel(mbconv_kernel<2, false>, grid, dim3(256), stream, ev, q);
}

}  // namespace lop
