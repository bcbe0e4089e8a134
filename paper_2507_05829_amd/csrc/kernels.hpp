// Launch interface of the gfx950 kernels. Every kernel works on row slabs: a tensor is
// N x rows x W x C (NHWC) holding rows [row0, row0 + rows) of an image of height h.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstddef>
#include <cstdint>

namespace lop {

struct Slab {
  void* ptr = nullptr;
  int n = 0, h = 0, w = 0, c = 0;  // h: true image height
  int row0 = 0, rows = 0;          // rows held
};

// One local operator on output rows [out_lo, out_hi): y = act(op(x) + bias + res).
struct OpLaunch {
  int op = 0;     // lop_op_t
  int dtype = 0;  // lop_dtype_t
  Slab x, y, res; // res.ptr == nullptr: no residual
  void* y2 = nullptr;  // optional second destination laid out exactly like y (mapped host
                       // memory): every output element is stored to both
  const void* w = nullptr;      // device, kernel layout (see pack_* below)
  const void* wd = nullptr;     // dense conv: the weights in operand order, or nullptr
  const void* wd16 = nullptr;   // dense conv: ... in the operand order of 16 x 16 tiles, or nullptr
  const void* wstem = nullptr;  // dense conv over very few input channels: fp32 weights
                                // [c_out / 4][k][4] for the first-layer kernel, or nullptr
  const float* bias = nullptr;  // device or nullptr
  int kh = 1, kw = 1, sh = 1, sw = 1, ph = 0, pw = 0, dh = 1, dw = 1;
  int act = 0;
  int out_lo = 0, out_hi = 0;
  int k_pad = 0;  // dense conv: padded reduction length of the packed weight rows
  void* ws = nullptr;  // dense conv: device scratch for split-K partial sums (may be null
                       // only if conv_workspace_bytes() is 0 for this launch)
};

// Dense conv weights are packed as [c_out_pad][k_pad], k = (a*kw + b)*c_in + ci, zero
// padded so the kernel never guards weight loads (every launch checks on the host that its
// channel tiles end inside c_out_pad).
// Layers whose c_in and c_out are multiples of the 16-byte vector get a second packing in
// MFMA operand order for the small-layer kernel: [c_out_pad / 32][k_pad / MK][64 lanes] x 16
// bytes, MK = 2 vectors of elements; lane = half*32 + (co % 32) holds
// w[co][step*MK + half*KE ... + KE) of the first packing. A third one serves 16 x 16 tiles:
// [c_out_pad / 16][k_pad / MK16][64 lanes] x 16 bytes, MK16 = 4 vectors, lane = quarter*16 +
// (co % 16) holds w[co][step*MK16 + quarter*KE ... + KE).
// The row count is padded to the widest channel tile that can take the layer: 128, and 256 once
// there are more than 128 channels (the 256-wide tile is never chosen below that), so the last
// channel tile of any kernel reads rows that exist.
constexpr int kConvCoutPad = 128;
int conv_k_pad(int c_in, int kh, int kw, int dtype);
inline int conv_cout_pad(int c_out) {
  const int unit = c_out > kConvCoutPad ? 2 * kConvCoutPad : kConvCoutPad;
  return (c_out + unit - 1) / unit * unit;
}

// Bytes of split-K scratch the dense conv launch needs (0: none).
size_t conv_workspace_bytes(const OpLaunch& L);
// True when a 1x1 dense conv takes the streaming kernel (which needs no workspace).
bool pointwise_applies(const OpLaunch& L);

// Events that time the kernels of one operator: pair 0 the operator's kernel, pair 1 the
// finish kernel of a dense conv whose reduction axis is cut into slices. `n` counts the
// pairs a launch has used.
struct KernelEvents {
  static constexpr int kMax = 2;
  hipEvent_t start[kMax] = {nullptr, nullptr}, stop[kMax] = {nullptr, nullptr};
  int n = 0;
};

// Enqueue the kernel(s) for one operator on `stream`; `ev` (optional) times them.
hipError_t launch_op(const OpLaunch& L, hipStream_t stream, KernelEvents* ev = nullptr);
// The same operator on several bands of one layer as one launch (the operation batching of
// Sec. IV-D): n descriptors that differ in slabs and rows only; bands that compute nothing are
// skipped. op_batchable: whether the operator's kernel has such a form (the 1x1 streaming kernel
// and the register-blocked depthwise kernel take one band at a time).
constexpr int kMaxBandsPerLaunch = 16;
bool op_batchable(const OpLaunch& L);
hipError_t launch_op_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev = nullptr);
int describe_op_bands(const OpLaunch* Ls, int n, char* name, size_t size);
size_t conv_workspace_bytes_bands(const OpLaunch* Ls, int n);
hipError_t launch_convpool_bands(const OpLaunch* convs, const OpLaunch* pools, int n, hipStream_t stream,
                                 KernelEvents* ev = nullptr);
int convpool_describe_bands(const OpLaunch* convs, const OpLaunch* pools, int n, char* name, size_t size);
// Whether launch_op's kernel for this operator honours OpLaunch::y2.
bool stores_second_output(const OpLaunch& L);
// The first-layer kernel (very few input channels, a short reduction axis, vector ALUs):
// whether a layer of this shape gets the packing it needs, whether a launch takes it, the
// launch and its kernel name.
bool stem_shape_applies(int c_in, int c_out, int kh, int kw, int sw, int dh, int dw, bool residual);
bool stem_applies(const OpLaunch& L);
hipError_t launch_stem(const OpLaunch& L, hipStream_t stream, KernelEvents* ev = nullptr);
int stem_describe(const OpLaunch& L, char* name, size_t size);
int stem_describe_bands(const OpLaunch* Ls, int n, char* name, size_t size);
// A dense convolution and the 2 x 2 stride-2 max pooling that reads it, as one launch: whether
// the pair qualifies (descriptors without slabs suffice), the launch (conv: input slab, weights,
// hyper-parameters; pool: output slab, y2 and the pooled rows out_lo..out_hi) and its kernel name.
bool convpool_applies(const OpLaunch& conv, const OpLaunch& pool);
bool convpool_pays(const OpLaunch& conv);  // for one launch of the conv alone (rows and slab geometry set)
hipError_t launch_convpool(const OpLaunch& conv, const OpLaunch& pool, hipStream_t stream,
                           KernelEvents* ev = nullptr);
int convpool_describe(const OpLaunch& conv, const OpLaunch& pool, char* name, size_t size);
// Name of the kernel instance launch_op would pick, as a profiler prints it (without the
// namespace and argument list), written to name[size]. Returns the number of K slices
// (1: a single kernel; > 1: followed by splitk_finish_kernel).
int describe_op(const OpLaunch& L, char* name, size_t size);

}  // namespace lop
