// C ABI of the library: plan construction (host planning + weight upload), the per-band
// scheduler (compute stream + copy stream + one event per band) and the queries.
#include <hip/hip_runtime.h>

#include <cstdint>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "devmem.hpp"
#include "kernels.hpp"
#include "lop.h"
#include "plan_state.hpp"
#include "plan_tables.hpp"

namespace lop {
hipError_t launch_conv_igemm(const OpLaunch& L, hipStream_t stream, KernelEvents* ev);
hipError_t launch_rowwise_op(const OpLaunch& L, hipStream_t stream, KernelEvents* ev);
hipError_t launch_copy_rows(void* dst, const void* src, size_t pitch, size_t len, int n,
                            hipStream_t stream, int workgroups);
hipError_t launch_fill_words(void* dst, size_t bytes, unsigned word, hipStream_t stream);

hipError_t launch_pointwise(const OpLaunch& L, hipStream_t stream, KernelEvents* ev);
bool mbconv_applies(const OpLaunch& e, const OpLaunch& d, const OpLaunch& p);
int mbconv_describe(const OpLaunch& d, const OpLaunch& p, char* name, size_t size);
hipError_t launch_mbconv(const OpLaunch& e, const OpLaunch& d, const OpLaunch& p, hipStream_t stream,
                         KernelEvents* ev);
int pointwise_describe(const OpLaunch& L, char* name, size_t size);
int conv_igemm_describe(const OpLaunch& L, char* name, size_t size);
int rowwise_describe(const OpLaunch& L, char* name, size_t size);
hipError_t launch_conv_igemm_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev);
int conv_igemm_describe_bands(const OpLaunch* Ls, int n, char* name, size_t size);
hipError_t launch_rowwise_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev);
bool rowwise_batchable(const OpLaunch& L);
hipError_t launch_stem_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev);

hipError_t launch_op(const OpLaunch& L, hipStream_t stream, KernelEvents* ev) {
  if (L.out_hi <= L.out_lo) return hipSuccess;
  if (L.op == LOP_CONV2D) {
    if (stem_applies(L)) return launch_stem(L, stream, ev);
    return pointwise_applies(L) ? launch_pointwise(L, stream, ev) : launch_conv_igemm(L, stream, ev);
  }
  return launch_rowwise_op(L, stream, ev);
}

bool stores_second_output(const OpLaunch& L) {
  return L.op != LOP_CONV2D || stem_applies(L) || !pointwise_applies(L);
}

bool op_batchable(const OpLaunch& L) {
  if (L.op == LOP_CONV2D) return stem_applies(L) || !pointwise_applies(L);
  return rowwise_batchable(L);
}

hipError_t launch_op_bands(const OpLaunch* Ls, int n, hipStream_t stream, KernelEvents* ev) {
  if (n < 1 || n > kMaxBandsPerLaunch) return hipErrorInvalidValue;
  if (n == 1) return launch_op(Ls[0], stream, ev);
  if (!op_batchable(Ls[0])) return hipErrorInvalidValue;
  if (Ls[0].op == LOP_CONV2D)
    return stem_applies(Ls[0]) ? launch_stem_bands(Ls, n, stream, ev) : launch_conv_igemm_bands(Ls, n, stream, ev);
  return launch_rowwise_bands(Ls, n, stream, ev);
}

int describe_op_bands(const OpLaunch* Ls, int n, char* name, size_t size) {
  if (n > 1 && Ls[0].op == LOP_CONV2D && stem_applies(Ls[0])) return stem_describe_bands(Ls, n, name, size);
  if (n == 1 || Ls[0].op != LOP_CONV2D) {
    const int k = describe_op(Ls[0], name, size);
    if (n > 1 && name && size) {   // the form that takes several bands carries _bands in its name
      std::string s(name);
      const size_t at = s.find('<');
      s.insert(at == std::string::npos ? s.size() : at, "_bands");
      snprintf(name, size, "%s", s.c_str());
    }
    return k;
  }
  return conv_igemm_describe_bands(Ls, n, name, size);
}

int describe_op(const OpLaunch& L, char* name, size_t size) {
  if (L.op != LOP_CONV2D) return rowwise_describe(L, name, size);
  if (stem_applies(L)) return stem_describe(L, name, size);
  return pointwise_applies(L) ? pointwise_describe(L, name, size) : conv_igemm_describe(L, name, size);
}
}  // namespace lop

// Scratch of lop_run_chain_static: the slabs of one band at a time and the split-K partial sums
// of one launch at a time, in an array that is part of the loaded code object instead of an
// allocation. Every GPU the library runs on holds its own copy, at its own address, until the
// process ends. In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[LOP_STATIC_SCRATCH_BYTES];

namespace {
thread_local int g_last_hip = 0;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once known

// Looks up the address of `scratch` on `device`, which must be the current device. Called when
// a plan is set up on a device, so that lop_run_chain_static itself makes no runtime query.
hipError_t resolve_static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[device]) return hipSuccess;
  void* ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  g_scratch_ptr[device] = ptr;
  return hipSuccess;
}

void* static_scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  return g_scratch_ptr[device];
}
}  // namespace

namespace lop {
int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return e == hipErrorOutOfMemory ? LOP_ERR_OOM : LOP_ERR_HIP;
}
}  // namespace lop

namespace {
using lop::hip_fail;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

namespace {

int upload_weights(lop_plan_t* P) {
  const lop::Tables& t = P->t;
  const int nl = t.n_layers();
  const bool bf = t.in.dtype == LOP_BF16;
  P->d_w.assign(nl, nullptr);
  P->d_wd.assign(nl, nullptr);
  P->d_wd16.assign(nl, nullptr);
  P->d_wstem.assign(nl, nullptr);
  P->d_bias.assign(nl, nullptr);
  for (int l = 0; l < nl; ++l) {
    const lop::LayerInfo& L = t.layers[l];
    const lop_layer_t& d = L.d;
    if (d.op == LOP_CONV2D) {
      if (!d.weight) return LOP_ERR_INVALID_ARG;
      const int kp = P->k_pad[l];
      const int cp = lop::conv_cout_pad(d.c_out);
      const size_t esz = t.esz();
      std::vector<unsigned char> host((size_t)cp * kp * esz, 0);
      // OIHW -> [co][ (a*kw + b)*c_in + ci ]
      for (int co = 0; co < d.c_out; ++co)
        for (int ci = 0; ci < d.c_in; ++ci)
          for (int a = 0; a < d.kh; ++a)
            for (int b = 0; b < d.kw; ++b) {
              const size_t src = (((size_t)co * d.c_in + ci) * d.kh + a) * d.kw + b;
              const size_t dst = (size_t)co * kp + (size_t)(a * d.kw + b) * d.c_in + ci;
              std::memcpy(&host[dst * esz], (const unsigned char*)d.weight + src * esz, esz);
            }
      LOP_HIP(lop::dev_alloc(&P->d_w[l], host.size()));
      LOP_HIP(hipMemcpy(P->d_w[l], host.data(), host.size(), hipMemcpyHostToDevice));
      if (P->has_wstem[l]) {
        // fp32 [c_out / 4][k][4] and, behind it, [c_out / 16][k][16], k = (a*kw + b)*c_in + ci:
        // four (sixteen) weights of one reduction element lie together at an address a whole
        // wavefront shares
        const size_t K = (size_t)d.c_in * d.kh * d.kw;
        std::vector<float> q(2 * (size_t)d.c_out * K);
        for (int co = 0; co < d.c_out; ++co)
          for (size_t k = 0; k < K; ++k) {
            float v;
            const unsigned char* src = &host[((size_t)co * kp + k) * esz];
            if (bf) {
              unsigned short h;
              std::memcpy(&h, src, 2);
              const unsigned u = (unsigned)h << 16;
              std::memcpy(&v, &u, 4);
            } else {
              std::memcpy(&v, src, 4);
            }
            q[((size_t)(co / 4) * K + k) * 4 + co % 4] = v;
            q[(size_t)d.c_out * K + ((size_t)(co / 16) * K + k) * 16 + co % 16] = v;
          }
        LOP_HIP(lop::dev_alloc(&P->d_wstem[l], q.size() * 4));
        LOP_HIP(hipMemcpy(P->d_wstem[l], q.data(), q.size() * 4, hipMemcpyHostToDevice));
      }
      const int ke = 16 / (int)esz;
      if (P->has_wd[l]) {
        // the same values in MFMA operand order: [co / 32][step][half*32 + co % 32] x 16 B
        std::vector<unsigned char> ord(host.size());
        const size_t steps = (size_t)kp / (2 * ke);
        for (int co = 0; co < cp; ++co)
          for (size_t st = 0; st < steps; ++st)
            for (int half = 0; half < 2; ++half) {
              const size_t src = (size_t)co * kp + st * 2 * ke + (size_t)half * ke;
              const size_t dst = (((size_t)(co / 32) * steps + st) * 64 + half * 32 + co % 32) * ke;
              std::memcpy(&ord[dst * esz], &host[src * esz], 16);
            }
        LOP_HIP(lop::dev_alloc(&P->d_wd[l], ord.size()));
        LOP_HIP(hipMemcpy(P->d_wd[l], ord.data(), ord.size(), hipMemcpyHostToDevice));
        if (P->has_wd16[l]) {
          // ... and in the order of 16 x 16 tiles: [co / 16][step][quarter*16 + co % 16] x 16 B
          const size_t steps16 = (size_t)kp / (4 * ke);
          for (int co = 0; co < cp; ++co)
            for (size_t st = 0; st < steps16; ++st)
              for (int q = 0; q < 4; ++q) {
                const size_t src = (size_t)co * kp + st * 4 * ke + (size_t)q * ke;
                const size_t dst = (((size_t)(co / 16) * steps16 + st) * 64 + q * 16 + co % 16) * ke;
                std::memcpy(&ord[dst * esz], &host[src * esz], 16);
              }
          LOP_HIP(lop::dev_alloc(&P->d_wd16[l], ord.size()));
          LOP_HIP(hipMemcpy(P->d_wd16[l], ord.data(), ord.size(), hipMemcpyHostToDevice));
        }
      }
    } else if (d.op == LOP_DWCONV2D) {
      if (!d.weight) return LOP_ERR_INVALID_ARG;
      // C x 1 x kh x kw (storage type) -> [tap][C] fp32
      std::vector<float> host((size_t)d.kh * d.kw * d.c_in);
      for (int c = 0; c < d.c_in; ++c)
        for (int tap = 0; tap < d.kh * d.kw; ++tap) {
          const size_t src = (size_t)c * d.kh * d.kw + tap;
          float v;
          if (bf) {
            const unsigned u = (unsigned)((const unsigned short*)d.weight)[src] << 16;
            std::memcpy(&v, &u, 4);
          } else {
            v = ((const float*)d.weight)[src];
          }
          host[(size_t)tap * d.c_in + c] = v;
        }
      LOP_HIP(lop::dev_alloc(&P->d_w[l], host.size() * 4));
      LOP_HIP(hipMemcpy(P->d_w[l], host.data(), host.size() * 4, hipMemcpyHostToDevice));
    }
    if (d.bias && d.op != LOP_MAXPOOL2D) {
      LOP_HIP(lop::dev_alloc((void**)&P->d_bias[l], (size_t)d.c_out * 4));
      LOP_HIP(hipMemcpy(P->d_bias[l], d.bias, (size_t)d.c_out * 4, hipMemcpyHostToDevice));
    }
  }
  return LOP_OK;
}

void size_scratch(lop_plan_t* P) {
  const lop::Tables& t = P->t;
  const int nl = t.n_layers();
  P->slab_off.assign(t.n_bands, std::vector<size_t>(nl, 0));
  size_t worst = 0;
  if (t.reuse) {
    // bands share one full-height buffer per layer (rows at their absolute position)
    size_t off = 0;
    for (int l = 0; l + 1 < nl; ++l) {
      for (int b = 0; b < t.n_bands; ++b) P->slab_off[b][l] = off;
      if (P->fused_away[l]) continue;
      off += align_up((size_t)t.in.n * t.layers[l].h_out * t.row_elems(l) * t.esz(), 256);
    }
    worst = off;
  } else {
    size_t base = 0;
    for (int b = 0; b < t.n_bands; ++b) {
      // (with batched launches all bands' slabs are live at once: one band's follow the other's)
      size_t off = P->batched ? base : 0;
      for (int l = 0; l + 1 < nl; ++l) {  // the last layer writes the caller's output
        const lop_rows_t r = t.bands[b].need[l + 1];
        P->slab_off[b][l] = off;
        if (r.hi > r.lo && !P->fused_away[l])
          off += align_up((size_t)t.in.n * (r.hi - r.lo) * t.row_elems(l) * t.esz(), 256);
      }
      worst = off > worst ? off : worst;
      base = off;
    }
  }
  P->arena_bytes = worst;
}

lop::OpLaunch make_launch(const lop_plan_t* P, int band, int l, const void* d_in, void* d_out);

// Largest split-K workspace any launch of the plan needs (the launch descriptors only need
// sizes here, not the scratch addresses).
void size_workspace(lop_plan_t* P) {
  P->conv_ws_bytes = 0;
  for (int b = 0; b < P->t.n_bands; ++b)
    for (int l = 0; l < P->t.n_layers(); ++l) {
      if (P->t.layers[l].d.op != LOP_CONV2D || P->fused_away[l] || P->fuse_head[l] >= 0) continue;
      const lop_rows_t rr = P->t.bands[b].compute[l];
      if (rr.hi <= rr.lo) continue;
      const lop::OpLaunch o = make_launch(P, b, l, nullptr, nullptr);
      const size_t need = lop::pointwise_applies(o) ? 0 : lop::conv_workspace_bytes(o);
      P->conv_ws_bytes = std::max(need, P->conv_ws_bytes);
    }
  if (P->batched)   // a layer's launch for all bands keeps every band's partial sums at once
    for (int l = 0; l < P->t.n_layers(); ++l) {
      if (P->t.layers[l].d.op != LOP_CONV2D || P->fused_away[l] || P->fuse_head[l] >= 0) continue;
      std::vector<lop::OpLaunch> group;
      for (int b = 0; b < P->t.n_bands; ++b) {
        const lop_rows_t rr = P->t.bands[b].compute[l];
        if (rr.hi > rr.lo) group.push_back(make_launch(P, b, l, nullptr, nullptr));
      }
      if (group.empty() || lop::pointwise_applies(group[0])) continue;
      P->conv_ws_bytes = std::max(lop::conv_workspace_bytes_bands(group.data(), (int)group.size()), P->conv_ws_bytes);
    }
}

// Whether every launch of the plan has a kernel form that takes several bands.
bool all_launches_batchable(const lop_plan_t* P) {
  const lop::Tables& t = P->t;
  if (t.n_bands > lop::kMaxBandsPerLaunch) return false;
  for (int l = 0; l < t.n_layers(); ++l) {
    if (P->fused_away[l]) continue;
    if (P->fuse_head[l] >= 0) {
      if (P->fuse_head[l] != l - 1) return false;   // an inverted-residual block
      continue;
    }
    if (!lop::op_batchable(lop::describe_layer(P, l))) return false;
  }
  return true;
}

lop::Slab slab_of(const lop_plan_t* P, int band, int tensor, const void* d_in, void* d_out) {
  const lop::Tables& t = P->t;
  const int nl = t.n_layers();
  lop::Slab s;
  s.n = t.in.n;
  s.h = t.tensor_h(tensor);
  if (tensor < 0) {
    s.ptr = const_cast<void*>(d_in);
    s.w = t.in.w; s.c = t.in.c; s.row0 = 0; s.rows = t.in.h;
  } else {
    s.w = t.layers[tensor].w_out;
    s.c = t.layers[tensor].d.c_out;
    if (tensor == nl - 1) {
      s.ptr = d_out; s.row0 = 0; s.rows = s.h;
    } else {
      // (no arena yet while the plan is being sized, and none at all in a plan-only plan)
      char* const arena = (char*)P->arena_of(band);
      s.ptr = arena ? arena + P->slab_off[band][tensor] : nullptr;
      if (t.reuse) {
        s.row0 = 0; s.rows = s.h;
      } else {
        const lop_rows_t r = t.bands[band].need[tensor + 1];
        s.row0 = r.lo; s.rows = r.hi - r.lo;
      }
    }
  }
  return s;
}

lop::OpLaunch make_launch(const lop_plan_t* P, int band, int l, const void* d_in, void* d_out) {
  const lop::Tables& t = P->t;
  const lop::LayerInfo& L = t.layers[l];
  lop::OpLaunch o;
  o.op = L.d.op;
  o.dtype = t.in.dtype;
  o.x = slab_of(P, band, L.d.input_from, d_in, d_out);
  o.y = slab_of(P, band, l, d_in, d_out);
  if (L.d.residual_from != LOP_NO_RESIDUAL) o.res = slab_of(P, band, L.d.residual_from, d_in, d_out);
  if (!P->d_w.empty()) {  // uploaded (a plan-only plan has tables but no device arrays)
    o.w = P->d_w[l];
    o.wd = P->d_wd[l];
    o.wd16 = P->d_wd16[l];
    o.wstem = P->d_wstem[l];
    o.bias = P->d_bias[l];
  } else {
    // not uploaded (yet): the kernel choice only asks which packings exist, so a marker that
    // is never dereferenced stands for each that upload_weights would make
    o.wd = P->has_wd[l] ? (const void*)P : nullptr;
    o.wd16 = P->has_wd16[l] ? (const void*)P : nullptr;
    o.wstem = P->has_wstem[l] ? (const void*)P : nullptr;
  }
  o.k_pad = P->k_pad[l];
  o.kh = L.d.kh; o.kw = L.d.kw; o.sh = L.d.sh; o.sw = L.d.sw;
  o.ph = L.d.ph; o.pw = L.d.pw; o.dh = L.d.dh; o.dw = L.d.dw;
  o.act = L.d.act;
  o.out_lo = t.bands[band].compute[l].lo;
  o.out_hi = t.bands[band].compute[l].hi;
  o.ws = P->ws_of(band);
  return o;
}

}  // namespace

namespace lop {
OpLaunch describe_layer(const lop_plan_s* P, int l) {
  const lop::LayerInfo& L = P->t.layers[l];
  lop::OpLaunch o;
  o.op = L.d.op;
  o.dtype = P->t.in.dtype;
  o.x.c = L.d.c_in; o.y.c = L.d.c_out;
  o.x.n = o.y.n = P->t.in.n;
  if (L.d.residual_from != LOP_NO_RESIDUAL) o.res.ptr = const_cast<lop_plan_t*>(P);
  if (!P->d_w.empty()) {  // uploaded (not a plan-only plan)
    o.w = P->d_w[l]; o.wd = P->d_wd[l]; o.wd16 = P->d_wd16[l]; o.wstem = P->d_wstem[l]; o.bias = P->d_bias[l];
  } else {
    o.wd = P->has_wd[l] ? (const void*)P : nullptr;
    o.wd16 = P->has_wd16[l] ? (const void*)P : nullptr;
    o.wstem = P->has_wstem[l] ? (const void*)P : nullptr;
  }
  o.k_pad = P->k_pad[l];
  o.kh = L.d.kh; o.kw = L.d.kw; o.sh = L.d.sh; o.sw = L.d.sw;
  o.ph = L.d.ph; o.pw = L.d.pw; o.dh = L.d.dh; o.dw = L.d.dw;
  o.act = L.d.act;
  return o;
}
}  // namespace lop

namespace {
using lop::describe_layer;

// Groups of three layers that run as one launch (an inverted-residual block): layer h a 1x1
// conv, h + 1 a depthwise conv reading only h, h + 2 a 1x1 conv reading only h + 1, and
// nobody else reads h or h + 1.
void find_fused_groups(lop_plan_t* P) {
  const lop::Tables& t = P->t;
  const int nl = t.n_layers();
  P->fuse_head.assign(nl, -1);
  P->fused_away.assign(nl, 0);
  if (P->flags & (LOP_FLAG_NO_FUSE | LOP_FLAG_PLAN_ONLY)) return;
  for (int h = 0; h + 2 < nl; ++h) {
    if (P->fused_away[h] || P->fuse_head[h] >= 0) continue;
    const int m = h + 1, q = h + 2;
    if (t.layers[m].d.input_from != h || t.layers[q].d.input_from != m) continue;
    bool shared = false;
    for (int j = 0; j < nl; ++j) {
      const lop_layer_t& d = t.layers[j].d;
      if (j != m && d.input_from == h) shared = true;
      if (j != q && d.input_from == m) shared = true;
      if (d.residual_from == h || d.residual_from == m) shared = true;
    }
    if (shared) continue;
    if (!lop::mbconv_applies(describe_layer(P, h), describe_layer(P, m), describe_layer(P, q))) continue;
    P->fuse_head[q] = h;
    P->fused_away[h] = P->fused_away[m] = 1;
    h = q;
  }
  // Groups of two: a dense conv and the 2 x 2 stride-2 max pooling that is its only reader.
  // The pooling windows do not overlap, so the rows of the conv a band computes are exactly
  // twice its pooled rows, in both modes (checked, since the launch derives them that way).
  for (int h = 0; h + 1 < nl; ++h) {
    const int q = h + 1;
    if (P->fused_away[h] || P->fuse_head[h] >= 0 || P->fused_away[q] || P->fuse_head[q] >= 0) continue;
    if (t.layers[q].d.input_from != h) continue;
    bool shared = false;
    for (int j = 0; j < nl; ++j) {
      const lop_layer_t& d = t.layers[j].d;
      if (j != q && d.input_from == h) shared = true;
      if (d.residual_from == h) shared = true;
    }
    if (shared) continue;
    if (!lop::convpool_applies(describe_layer(P, h), describe_layer(P, q))) continue;
    const lop::LayerInfo& C = t.layers[h];
    const size_t esz = t.esz();
    if ((size_t)C.n * C.h_in * C.w_in * C.d.c_in * esz >= ((size_t)1 << 31)) continue;  // 32-bit offsets
    bool rows_match = true;
    for (int b = 0; b < t.n_bands; ++b) {
      const lop_rows_t pr = t.bands[b].compute[q], cr = t.bands[b].compute[h];
      if (pr.hi <= pr.lo) rows_match = rows_match && cr.hi <= cr.lo;
      else rows_match = rows_match && cr.lo == 2 * pr.lo && cr.hi == 2 * pr.hi &&
                        lop::convpool_pays(make_launch(P, b, h, nullptr, nullptr));
    }
    if (!rows_match) continue;
    P->fuse_head[q] = h;
    P->fused_away[h] = 1;
  }
}

// Whether layer l ends a conv + pooling group (else, if it ends a group, an inverted-residual block).
bool ends_convpool(const lop_plan_t* P, int l) { return P->fuse_head[l] >= 0 && P->fuse_head[l] == l - 1; }

// The two descriptors of a conv + pooling launch of one band.
void convpool_launches(const lop_plan_t* P, int band, int l, const void* d_in, void* d_out,
                       lop::OpLaunch* conv, lop::OpLaunch* pool) {
  const int h = P->fuse_head[l];
  *pool = make_launch(P, band, l, d_in, d_out);
  *conv = make_launch(P, band, h, d_in, d_out);   // (its y slab is never used: the layer has no buffer)
}

// Rows of layer l one launch of band `band` produces (none for a layer that is part of a
// later layer's launch).
lop_rows_t launch_rows(const lop_plan_t* P, int band, int l) {
  if (P->fused_away[l]) return lop_rows_t{0, 0};
  return P->t.bands[band].compute[l];
}

// Enqueue what produces layer l's rows of one band: its own kernel(s), or the fused launch
// of the group it ends.
hipError_t launch_layer(const lop_plan_t* P, int band, int l, const void* d_in, void* d_out,
                        hipStream_t cs, lop::KernelEvents* ev = nullptr, void* y2 = nullptr) {
  const lop_rows_t r = launch_rows(P, band, l);
  if (r.hi <= r.lo) return hipSuccess;
  if (P->fuse_head[l] < 0) {
    lop::OpLaunch o = make_launch(P, band, l, d_in, d_out);
    o.y2 = y2;
    return lop::launch_op(o, cs, ev);
  }
  if (ends_convpool(P, l)) {
    lop::OpLaunch conv, pool;
    convpool_launches(P, band, l, d_in, d_out, &conv, &pool);
    pool.y2 = y2;
    return lop::launch_convpool(conv, pool, cs, ev);
  }
  const int h = P->fuse_head[l];
  lop::OpLaunch e = describe_layer(P, h), d = describe_layer(P, h + 1);
  const lop::OpLaunch p = make_launch(P, band, l, d_in, d_out);
  e.x = slab_of(P, band, P->t.layers[h].d.input_from, d_in, d_out);
  return lop::launch_mbconv(e, d, p, cs, ev);
}

// Kernel name (and reduction slices) of that launch.
int describe_layer_launch(const lop_plan_t* P, int band, int l, char* name, size_t size) {
  const lop_rows_t r = launch_rows(P, band, l);
  if (r.hi <= r.lo) return 0;
  if (P->fuse_head[l] < 0) return lop::describe_op(make_launch(P, band, l, nullptr, nullptr), name, size);
  if (ends_convpool(P, l)) {
    lop::OpLaunch conv, pool;
    convpool_launches(P, band, l, nullptr, nullptr, &conv, &pool);
    return lop::convpool_describe(conv, pool, name, size);
  }
  return lop::mbconv_describe(describe_layer(P, l - 1), describe_layer(P, l), name, size);
}

// Algorithmic work of that launch. A fused group: the three layers' operations on the rows
// it computes (the expand layer on the input rows the depthwise windows touch), and the
// bytes of the group's input rows, output rows, residual and weights only.
void launch_work(const lop_plan_t* P, int band, int l, double* flop, double* bytes) {
  const lop::Tables& t = P->t;
  const lop_rows_t r = launch_rows(P, band, l);
  *flop = 0.0;
  *bytes = 0.0;
  if (r.hi <= r.lo) return;
  if (P->fuse_head[l] < 0) {
    *flop = t.layer_flop(l, r.hi - r.lo);
    *bytes = t.layer_bytes(band, l);
    return;
  }
  if (ends_convpool(P, l)) {
    // the conv's operations on twice the pooled rows plus the comparisons; bytes of the conv's
    // input rows and weights and of the pooled rows only
    const int h = P->fuse_head[l];
    const lop::LayerInfo &C = t.layers[h], &Q = t.layers[l];
    const lop_rows_t rd = t.bands[band].reads[h];
    *flop = t.layer_flop(h, 2 * (r.hi - r.lo)) + t.layer_flop(l, r.hi - r.lo);
    const double e = (double)t.esz();
    *bytes = e * Q.n * ((double)(rd.hi - rd.lo) * C.w_in * C.d.c_in + (double)(r.hi - r.lo) * Q.w_out * Q.d.c_out) +
             e * (double)C.d.c_out * C.d.c_in * C.d.kh * C.d.kw;
    return;
  }
  const int h = P->fuse_head[l], m = h + 1;
  const lop::LayerInfo &E = t.layers[h], &D = t.layers[m], &Q = t.layers[l];
  const int in_lo = std::max(r.lo * D.d.sh - D.d.ph, 0);
  const int in_hi = std::min((r.hi - 1) * D.d.sh - D.d.ph + D.d.kh, D.h_in);
  const int rows_e = std::max(in_hi - in_lo, 0);
  *flop = t.layer_flop(l, r.hi - r.lo) + t.layer_flop(m, r.hi - r.lo) + t.layer_flop(h, rows_e);
  const double e = (double)t.esz();
  double b = e * Q.n * ((double)rows_e * E.w_in * E.d.c_in + (double)(r.hi - r.lo) * Q.w_out * Q.d.c_out);
  if (Q.d.residual_from != LOP_NO_RESIDUAL) b += e * Q.n * (double)(r.hi - r.lo) * Q.w_out * Q.d.c_out;
  b += e * ((double)E.d.c_out * E.d.c_in + 9.0 * D.d.c_out + (double)Q.d.c_out * Q.d.c_in);
  *bytes = b;
}

void* device_view_of_host(lop_plan_t* P, void* h_out);

// Small band outputs leave through the last layer's own stores: its kernel writes every
// element to the device tensor and to the mapped host buffer, so there is no copy launch to
// wait for on the lane. Larger outputs keep the paced copy kernel (stores over PCIe from a
// whole grid hold up the HBM writes of the kernels beside them).
constexpr size_t kDirectHostStoreMax = 256 * 1024;
// Workgroups of a band copy that shares a stream with kernels: its stores are paced by the
// link, and many of them in flight hold up the HBM writes of the kernels running beside the
// copy (4 workgroups move about 30 GB/s; with 64 the copy was 1.7x faster and the other
// streams lost more than that; on a lane of its own 8 and 16 workgroups cost the chains beside
// it 8 % and 13 %).
constexpr int kCopyWorkgroups = 4;
constexpr size_t kCopyLaneMaxBytes = (size_t)64 << 20;

// Device view of h_out if band `band` can deliver its rows that way, else nullptr.
void* direct_host_target(lop_plan_t* P, int band, void* h_out) {
  if (!h_out || (P->flags & (LOP_FLAG_NO_D2H | LOP_FLAG_DMA_COPY))) return nullptr;
  const lop::Tables& t = P->t;
  const int last = t.n_layers() - 1;
  if (P->fuse_head[last] >= 0 && !ends_convpool(P, last)) return nullptr;
  const lop_rows_t r = t.bands[band].need[t.n_layers()];
  const size_t bytes = (size_t)t.in.n * (r.hi - r.lo) * t.row_elems(last) * t.esz();
  if (bytes == 0 || bytes > kDirectHostStoreMax) return nullptr;
  if (!ends_convpool(P, last) &&   // (the pooled launch stores to both destinations)
      !lop::stores_second_output(make_launch(P, band, last, nullptr, nullptr)))
    return nullptr;
  return device_view_of_host(P, h_out);
}

bool band_empty(const lop_plan_t* P, int band) {
  const lop_rows_t r = P->t.bands[band].need[P->t.n_layers()];
  return r.hi <= r.lo;
}

int enqueue_band_kernels(lop_plan_t* P, int band, const void* d_in, void* d_out, hipStream_t cs,
                         void* y2 = nullptr) {
  const int nl = P->t.n_layers();
  if (P->flags & LOP_FLAG_POISON_SCRATCH) {
    // Debug aid: every scratch byte the band could read is NaN (all bits set, in both storage
    // types) unless this band's own launches write it first, so a kernel that reads a row outside
    // the intervals the plan gave it shows up in the output. In reuse mode earlier bands' rows
    // are read on purpose: the slabs are poisoned once, before the chain's first band.
    bool first = true;
    for (int b = 0; b < band; ++b) first = first && band_empty(P, b);
    if (!P->t.reuse || first)
      LOP_HIP(lop::launch_fill_words(P->arena_of(band), align_up(P->arena_bytes, 256), 0xFFFFFFFFu, cs));
    LOP_HIP(lop::launch_fill_words(P->ws_of(band), P->conv_ws_bytes / 16 * 16, 0xFFFFFFFFu, cs));
  }
  for (int l = 0; l < nl; ++l)
    LOP_HIP(launch_layer(P, band, l, d_in, d_out, cs, nullptr, l == nl - 1 ? y2 : nullptr));
  return LOP_OK;
}

// Device-side address of a pinned, mapped host buffer, or nullptr if the buffer is not
// such memory. Looked up once per pointer.
void* device_view_of_host(lop_plan_t* P, void* h_out) {
  for (const auto& e : P->host_views)
    if (e.first == h_out) return e.second;
  void* dev = nullptr;
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, h_out) == hipSuccess) {
    if (attr.type == hipMemoryTypeHost && attr.devicePointer) dev = attr.devicePointer;
  } else {
    (void)hipGetLastError();  // pageable memory: clear the sticky error, use the DMA path
  }
  if (P->host_views.size() >= 16) P->host_views.erase(P->host_views.begin());
  P->host_views.emplace_back(h_out, dev);
  return dev;
}

// Copy the band's final rows of every image to the host buffer (same NHWC layout).
int enqueue_band_copy(lop_plan_t* P, int band, const void* d_out, void* h_out, hipStream_t s) {
  const lop::Tables& t = P->t;
  const lop_rows_t r = t.bands[band].need[t.n_layers()];
  if (r.hi <= r.lo) return LOP_OK;
  const lop::LayerInfo& L = t.layers.back();
  const size_t row_b = (size_t)t.row_elems(t.n_layers() - 1) * t.esz();
  const size_t img_b = row_b * L.h_out;
  const size_t off = row_b * r.lo, len = row_b * (r.hi - r.lo);
  // Mapped pinned host memory is written by a small kernel on the copy stream (no DMA
  // set-up cost per band, and it can be captured like any kernel); a plan made with
  // LOP_FLAG_DMA_COPY goes through the runtime's copy engines instead. Host memory that is
  // not pinned is refused (the boundary asks for pinned memory: an asynchronous copy into
  // pageable memory is staged by the runtime and is neither asynchronous nor cheap).
  void* mapped = device_view_of_host(P, h_out);
  if (!mapped) return LOP_ERR_INVALID_ARG;
  if (P->flags & LOP_FLAG_DMA_COPY) mapped = nullptr;
  if (mapped) {
    LOP_HIP(lop::launch_copy_rows((char*)mapped + off, (const char*)d_out + off, img_b, len,
                                  t.in.n, s, kCopyWorkgroups));
    return LOP_OK;
  }
  if (t.in.n == 1) {
    LOP_HIP(hipMemcpyAsync((char*)h_out + off, (const char*)d_out + off, len,
                           hipMemcpyDeviceToHost, s));
  } else {
    LOP_HIP(hipMemcpy2DAsync((char*)h_out + off, img_b, (const char*)d_out + off, img_b, len,
                             t.in.n, hipMemcpyDeviceToHost, s));
  }
  return LOP_OK;
}

int ensure_timing_events(lop_plan_t* P) {
  if (!P->ev_c0.empty()) return LOP_OK;
  const int nb = P->t.n_bands;
  for (auto* v : {&P->ev_c0, &P->ev_c1, &P->ev_d0, &P->ev_d1}) {
    v->assign(nb, nullptr);
    for (int b = 0; b < nb; ++b) LOP_HIP(hipEventCreate(&(*v)[b]));
  }
  LOP_HIP(hipEventCreate(&P->ev_t0));
  LOP_HIP(hipEventCreate(&P->ev_t1));
  return LOP_OK;
}

int setup_device(lop_plan_t* P) {
  LOP_HIP(hipGetDevice(&P->device));
  LOP_HIP(resolve_static_scratch(P->device));
  int rc = upload_weights(P);
  if (rc != LOP_OK) return rc;
  const int nb = P->t.n_bands;
  int live = 0;
  for (int b = 0; b < nb; ++b) live += band_empty(P, b) ? 0 : 1;
  int want = (int)((P->flags >> 8) & 0xff);
  if (want == 0) want = LOP_DEFAULT_LANES;
  const int n_lanes = P->t.reuse || P->batched ? std::max(1, want) : std::max(1, std::min(want, live));
  P->lanes.assign(n_lanes, Lane{});
  // Long band copies (stores into host memory, paced by the link) get a lane of their own.
  // On a compute lane a copy holds up that lane's next band, and because the bands are equal
  // the lanes reach their copies together: all of them copy at once, at the link's rate, with
  // nothing computing beside them, and then all compute at once with the link idle.
  size_t longest_copy = 0, all_copies = 0;
  for (int b = 0; b < nb; ++b) {
    const lop_rows_t r = P->t.bands[b].need[P->t.n_layers()];
    if (r.hi <= r.lo) continue;
    const size_t bytes = (size_t)P->t.in.n * (r.hi - r.lo) * P->t.row_elems(P->t.n_layers() - 1) * P->t.esz();
    longest_copy = std::max(longest_copy, bytes);
    all_copies += bytes;
  }
  // Independent bands only: in reuse mode a lane holds a whole chain, and three chains in
  // flight plus a copy lane measured slower than four chains that copy on their own lanes.
  // Not for chains whose result is so large that the copies, one after another at the copy
  // kernel's 30 GB/s, would take longer than the kernels (a matrix product chain with 134 MB of
  // output per call: 215 calls/s with the copy lane, 350 with copies on every lane, which
  // together reach the link's rate). The plan does not know the kernels' time; the bound on the
  // bytes stands for it.
  P->copy_lane = !P->t.reuse && !P->batched && n_lanes >= 3 && longest_copy > kDirectHostStoreMax &&
                 all_copies <= kCopyLaneMaxBytes &&
                 !(P->flags & (LOP_FLAG_NO_D2H | LOP_FLAG_DMA_COPY));
  for (Lane& L : P->lanes) {
    const bool computes = !P->copy_lane || &L != &P->lanes.back();
    if (P->arena_bytes && computes) LOP_HIP(lop::dev_alloc(&L.arena, align_up(P->arena_bytes, 256)));
    if (P->conv_ws_bytes && computes) {
      LOP_HIP(lop::dev_alloc(&L.conv_ws, P->conv_ws_bytes));
    }
    LOP_HIP(hipStreamCreateWithFlags(&L.stream, hipStreamNonBlocking));
    LOP_HIP(hipStreamCreateWithFlags(&L.copy, hipStreamNonBlocking));
    LOP_HIP(hipEventCreateWithFlags(&L.ev_join, hipEventDisableTiming));
  }
  LOP_HIP(hipStreamCreateWithFlags(&P->s_main, hipStreamNonBlocking));
  LOP_HIP(hipStreamCreateWithFlags(&P->s_copy, hipStreamNonBlocking));
  LOP_HIP(hipEventCreateWithFlags(&P->ev_fork, hipEventDisableTiming));
  LOP_HIP(hipEventCreateWithFlags(&P->ev_copy_tail, hipEventDisableTiming));
  P->ev_done.assign(nb, nullptr);
  P->ev_copied.assign(nb, nullptr);
  P->copied_valid.assign(nb, 0);
  for (auto& e : P->ev_done) LOP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  for (auto& e : P->ev_copied) LOP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  LOP_HIP(hipDeviceSynchronize());
  return LOP_OK;
}

// Kernels of one band on stream `cs`, then (optionally) its device-to-host copy on the
// copy stream, gated by the band's "kernels finished" event.
int enqueue_band(lop_plan_t* P, int band, const void* d_in, void* d_out, void* h_out,
                 hipStream_t cs, hipStream_t ds, bool timing, bool capturing = false) {
  // the band's rows of d_out may still be in flight to the host from an earlier call
  if (P->copied_valid[band] && !capturing)
    LOP_HIP(hipStreamWaitEvent(cs, P->ev_copied[band], 0));
  if (timing) LOP_HIP(hipEventRecord(P->ev_c0[band], cs));
  void* const direct = direct_host_target(P, band, h_out);
  int rc = enqueue_band_kernels(P, band, d_in, d_out, cs, direct);
  if (rc != LOP_OK) return rc;
  if (timing) LOP_HIP(hipEventRecord(P->ev_c1[band], cs));
  if (direct) {  // the rows are on their way already: nothing to copy, nothing to wait for
    if (timing) {
      LOP_HIP(hipEventRecord(P->ev_d0[band], cs));
      LOP_HIP(hipEventRecord(P->ev_d1[band], cs));
    }
    if (!capturing) {
      LOP_HIP(hipEventRecord(P->ev_copied[band], cs));
      P->copied_valid[band] = 1;
    }
  } else if (h_out && !(P->flags & LOP_FLAG_NO_D2H)) {
    if (ds != cs) {  // stream order already gates a copy on the kernels' own stream
      LOP_HIP(hipEventRecord(P->ev_done[band], cs));
      LOP_HIP(hipStreamWaitEvent(ds, P->ev_done[band], 0));
    }
    if (timing) LOP_HIP(hipEventRecord(P->ev_d0[band], ds));
    rc = enqueue_band_copy(P, band, d_out, h_out, ds);
    if (rc != LOP_OK) return rc;
    if (timing) LOP_HIP(hipEventRecord(P->ev_d1[band], ds));
    if (!capturing) {
      LOP_HIP(hipEventRecord(P->ev_copied[band], ds));
      P->copied_valid[band] = 1;
    }
  }
  return LOP_OK;
}

// Fork the lanes from `ms`, enqueue every band, join the lanes back into `ms`.
int enqueue_chain(lop_plan_t* P, const void* d_in, void* d_out, void* h_out, hipStream_t ms,
                  bool timing, bool capturing) {
  hipStream_t ds = P->s_copy;
  LOP_HIP(hipEventRecord(P->ev_fork, ms));
  for (Lane& L : P->lanes) LOP_HIP(hipStreamWaitEvent(L.stream, P->ev_fork, 0));
  bool copied = false;
  for (int b = 0; b < P->t.n_bands; ++b) {
    if (band_empty(P, b)) continue;
    // With several lanes a band's copy follows its kernels on the lane's own stream and
    // overlaps the other lanes' kernels; a single lane needs the separate copy stream to
    // overlap band b's copy with band b+1's kernels.
    hipStream_t cs = P->lane_of(b).stream;
    int rc = enqueue_band(P, b, d_in, d_out, h_out, cs, P->n_lanes() > 1 ? cs : ds, timing,
                          capturing);
    if (rc != LOP_OK) return rc;
    copied = copied || (h_out && !(P->flags & LOP_FLAG_NO_D2H));
  }
  // join: the main stream continues once every lane's kernels are done. Eagerly the
  // copies are not joined, so the last copy can run under whatever is enqueued next; a
  // captured graph has to join every stream it forked.
  for (Lane& L : P->lanes) {
    LOP_HIP(hipEventRecord(L.ev_join, L.stream));
    LOP_HIP(hipStreamWaitEvent(ms, L.ev_join, 0));
  }
  if (capturing && copied && P->n_lanes() == 1) {
    LOP_HIP(hipEventRecord(P->ev_copy_tail, ds));
    LOP_HIP(hipStreamWaitEvent(ms, P->ev_copy_tail, 0));
  }
  return LOP_OK;
}

// Bands of a reuse-mode chain, in order, on one lane.
int enqueue_chain_reuse(lop_plan_t* P, const void* d_in, void* d_out, void* h_out, bool timing,
                        bool capturing) {
  Lane& L = P->lanes[P->cur_lane];
  // With several lanes a band's copy follows its kernels on the lane and overlaps the
  // other lanes' chains (cross-stream edges inside a captured graph were measured to
  // serialise the lanes); a single lane uses its copy stream so that band b's copy
  // overlaps band b+1's kernels.
  hipStream_t ds = P->n_lanes() > 1 ? L.stream : L.copy;
  bool copied = false;
  for (int b = 0; b < P->t.n_bands; ++b) {
    if (band_empty(P, b)) continue;
    int rc = enqueue_band(P, b, d_in, d_out, h_out, L.stream, ds, timing, capturing);
    if (rc != LOP_OK) return rc;
    copied = copied || (h_out && !(P->flags & LOP_FLAG_NO_D2H));
  }
  if (capturing && copied && ds != L.stream) {  // a captured graph joins the stream it forked
    LOP_HIP(hipEventRecord(P->ev_copy_tail, ds));
    LOP_HIP(hipStreamWaitEvent(L.stream, P->ev_copy_tail, 0));
  }
  return LOP_OK;
}

// The descriptors of layer l's launch for all bands (convs: the conv of a conv + pooling group,
// else empty). y2 of band b is its direct host target when h_out is given (last layer only).
void batched_group(lop_plan_t* P, int l, const void* d_in, void* d_out, void* h_out,
                   std::vector<lop::OpLaunch>* group, std::vector<lop::OpLaunch>* convs,
                   std::vector<char>* direct) {
  group->clear();
  convs->clear();
  for (int b = 0; b < P->t.n_bands; ++b) {
    const lop_rows_t r = launch_rows(P, b, l);
    if (r.hi <= r.lo) continue;
    lop::OpLaunch o = make_launch(P, b, l, d_in, d_out);
    if (h_out) {
      o.y2 = direct_host_target(P, b, h_out);
      if (direct) (*direct)[b] = o.y2 != nullptr;
    }
    if (ends_convpool(P, l)) {
      lop::OpLaunch conv, pool;
      convpool_launches(P, b, l, d_in, d_out, &conv, &pool);
      pool.y2 = o.y2;
      convs->push_back(conv);
      group->push_back(pool);
    } else {
      group->push_back(o);
    }
  }
}

// One launch (plus its finish kernel, if the reduction is cut) for layer l of every band.
hipError_t launch_layer_batched(lop_plan_t* P, int l, const void* d_in, void* d_out, hipStream_t cs,
                                lop::KernelEvents* ev, void* h_out, std::vector<char>* direct) {
  if (P->fused_away[l]) return hipSuccess;
  std::vector<lop::OpLaunch> group, convs;
  batched_group(P, l, d_in, d_out, h_out, &group, &convs, direct);
  if (group.empty()) return hipSuccess;
  if (ends_convpool(P, l)) return lop::launch_convpool_bands(convs.data(), group.data(), (int)group.size(), cs, ev);
  return lop::launch_op_bands(group.data(), (int)group.size(), cs, ev);
}

// Kernel name and reduction slices of that launch.
int describe_layer_batched(const lop_plan_t* P, int l, char* name, size_t size) {
  if (P->fused_away[l]) return 0;
  std::vector<lop::OpLaunch> group, convs;
  batched_group(const_cast<lop_plan_t*>(P), l, nullptr, nullptr, nullptr, &group, &convs, nullptr);
  if (group.empty()) return 0;
  if (ends_convpool(P, l)) return lop::convpool_describe_bands(convs.data(), group.data(), (int)group.size(), name, size);
  return lop::describe_op_bands(group.data(), (int)group.size(), name, size);
}

// The band a batched plan's launch of layer l is attributed to in per-band queries: the first
// band that computes rows of it (-1: nobody does).
int batched_owner(const lop_plan_t* P, int l) {
  for (int b = 0; b < P->t.n_bands; ++b) {
    const lop_rows_t r = launch_rows(P, b, l);
    if (r.hi > r.lo) return b;
  }
  return -1;
}

// A chain whose launches are batched over the bands (Sec. IV-D operation batching), on one
// lane: per layer one launch that computes every band's rows on that band's slabs, then the
// bands' rows to the host (through the last launch's own stores where a band is small enough,
// else by copies behind it).
int enqueue_chain_batched(lop_plan_t* P, const void* d_in, void* d_out, void* h_out, bool timing,
                          bool capturing) {
  Lane& L = P->lanes[P->cur_lane];
  hipStream_t cs = L.stream;
  const int nb = P->t.n_bands, nl = P->t.n_layers();
  const bool copy = h_out && !(P->flags & LOP_FLAG_NO_D2H);
  if (!capturing)
    for (int b = 0; b < nb; ++b)
      if (P->copied_valid[b]) {  // these rows of d_out may still be on their way to the host
        LOP_HIP(hipStreamWaitEvent(cs, P->ev_copied[b], 0));
        P->copied_valid[b] = 0;
      }
  if (P->flags & LOP_FLAG_POISON_SCRATCH) {
    LOP_HIP(lop::launch_fill_words(P->arena_of(0), align_up(P->arena_bytes, 256), 0xFFFFFFFFu, cs));
    LOP_HIP(lop::launch_fill_words(P->ws_of(0), P->conv_ws_bytes / 16 * 16, 0xFFFFFFFFu, cs));
  }
  if (timing)
    for (int b = 0; b < nb; ++b)
      if (!band_empty(P, b)) LOP_HIP(hipEventRecord(P->ev_c0[b], cs));
  std::vector<char> direct(nb, 0);
  for (int l = 0; l < nl; ++l)
    LOP_HIP(launch_layer_batched(P, l, d_in, d_out, cs, nullptr, l == nl - 1 && copy ? h_out : nullptr, &direct));
  for (int b = 0; b < nb; ++b) {
    if (band_empty(P, b)) continue;
    if (timing) {
      LOP_HIP(hipEventRecord(P->ev_c1[b], cs));
      LOP_HIP(hipEventRecord(P->ev_d0[b], cs));
    }
    if (copy && !direct[b]) {
      int rc = enqueue_band_copy(P, b, d_out, h_out, cs);
      if (rc != LOP_OK) return rc;
    }
    if (timing) LOP_HIP(hipEventRecord(P->ev_d1[b], cs));
    if (copy && !capturing) {
      LOP_HIP(hipEventRecord(P->ev_copied[b], cs));
      P->copied_valid[b] = 1;
    }
  }
  return LOP_OK;
}

// The bands of lane `lane` of an independent-mode chain, in order, on that lane's stream.
int enqueue_lane(lop_plan_t* P, int lane, const void* d_in, void* d_out, void* h_out, bool capturing) {
  hipStream_t cs = P->lanes[lane].stream;
  for (int b = lane; b < P->t.n_bands; b += P->n_lanes()) {
    if (band_empty(P, b)) continue;
    int rc = enqueue_band(P, b, d_in, d_out, h_out, cs, cs, false, capturing);
    if (rc != LOP_OK) return rc;
  }
  return LOP_OK;
}

// lane_only >= 0 (independent mode): the graph holds that lane's bands only and runs on the
// lane's stream `ms`; -1: the whole chain forked from and joined into `ms`.
// band_only >= 0: the graph holds that band's kernels and nothing else (its copy is the
// caller's business).
int launch_graph(lop_plan_t* P, const void* d_in, void* d_out, void* h_out, hipStream_t ms,
                 int lane_only = -1, int band_only = -1) {
  const int lane = P->t.reuse || P->batched ? P->cur_lane : (lane_only >= 0 ? lane_only : -1);
  // an eager run may still have copies of the output rows in flight (on a copy stream that the
  // graph's stream is not ordered behind): a replay, and the first capture, wait for them
  for (int b = 0; b < P->t.n_bands; ++b)
    if (P->copied_valid[b] && (band_only < 0 || b == band_only)) {
      LOP_HIP(hipStreamWaitEvent(ms, P->ev_copied[b], 0));
      P->copied_valid[b] = 0;
    }
  for (const auto& g : P->graphs)
    if (g.d_in == d_in && g.d_out == d_out && g.h_out == h_out && g.lane == lane &&
        g.band == band_only) {
      LOP_HIP(hipGraphLaunch(g.exec, ms));
      return LOP_OK;
    }
  if (h_out) (void)device_view_of_host(P, h_out);  // query before capture starts
  hipGraph_t graph = nullptr;
  LOP_HIP(hipStreamBeginCapture(ms, hipStreamCaptureModeThreadLocal));
  int rc = band_only >= 0 ? enqueue_band_kernels(P, band_only, d_in, d_out, ms)
           : P->batched  ? enqueue_chain_batched(P, d_in, d_out, h_out, false, true)
           : P->t.reuse  ? enqueue_chain_reuse(P, d_in, d_out, h_out, false, true)
           : lane_only >= 0 ? enqueue_lane(P, lane_only, d_in, d_out, h_out, true)
                            : enqueue_chain(P, d_in, d_out, h_out, ms, false, true);
  hipError_t e = hipStreamEndCapture(ms, &graph);
  if (rc != LOP_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  if (e != hipSuccess) return hip_fail(e);
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return hip_fail(e);
  if (P->graphs.size() >= 128) {  // bounded cache: drop the oldest
    (void)hipGraphExecDestroy(P->graphs.front().exec);
    P->graphs.erase(P->graphs.begin());
  }
  P->graphs.push_back({d_in, d_out, h_out, lane, band_only, exec});
  LOP_HIP(hipGraphLaunch(exec, ms));
  return LOP_OK;
}

// Copy-lane schedule of one band: its kernels on compute stream `cs` (as a graph of their own
// when graphs are on), its copy on the copy lane behind the band's "kernels finished" event.
int enqueue_band_with_copy_lane(lop_plan_t* P, int band, const void* d_in, void* d_out,
                                void* h_out, hipStream_t cs) {
  hipStream_t ds = P->lanes.back().stream;
  int rc;
  if (P->flags & LOP_FLAG_GRAPH) {
    rc = launch_graph(P, d_in, d_out, nullptr, cs, P->lane_index(band), band);
  } else {
    if (P->copied_valid[band]) {  // these rows of d_out may still be on their way to the host
      LOP_HIP(hipStreamWaitEvent(cs, P->ev_copied[band], 0));
      P->copied_valid[band] = 0;
    }
    rc = enqueue_band_kernels(P, band, d_in, d_out, cs);
  }
  if (rc != LOP_OK) return rc;
  LOP_HIP(hipEventRecord(P->ev_done[band], cs));
  LOP_HIP(hipStreamWaitEvent(ds, P->ev_done[band], 0));
  rc = enqueue_band_copy(P, band, d_out, h_out, ds);
  if (rc != LOP_OK) return rc;
  LOP_HIP(hipEventRecord(P->ev_copied[band], ds));
  P->copied_valid[band] = 1;
  return LOP_OK;
}

}  // namespace

extern "C" {

int lop_plan(const lop_layer_t* layers, int n_layers, const lop_tensor_desc_t* in, int n_bands,
             unsigned flags, lop_plan_t** out_plan) {
  if (!out_plan) return LOP_ERR_INVALID_ARG;
  *out_plan = nullptr;
  lop_plan_t* P = new (std::nothrow) lop_plan_t;
  if (!P) return LOP_ERR_OOM;
  int rc = lop::build_tables(layers, n_layers, in, n_bands, (flags & LOP_FLAG_REUSE) != 0, P->t);
  if (rc != LOP_OK) { delete P; return rc; }
  P->flags = flags;
  P->k_pad.assign((size_t)n_layers, 0);  // padded reduction length of every dense conv
  P->has_wd.assign((size_t)n_layers, 0);
  P->has_wd16.assign((size_t)n_layers, 0);
  P->has_wstem.assign((size_t)n_layers, 0);
  const int ke = 16 / (int)P->t.esz();
  for (int l = 0; l < n_layers; ++l) {
    const lop_layer_t& d = P->t.layers[l].d;
    if (d.op != LOP_CONV2D) continue;
    P->k_pad[l] = lop::conv_k_pad(d.c_in, d.kh, d.kw, in->dtype);
    P->has_wd[l] = d.c_in % ke == 0 && d.c_out % ke == 0;
    P->has_wd16[l] = P->has_wd[l] && P->k_pad[l] % (4 * ke) == 0;
    P->has_wstem[l] = lop::stem_shape_applies(d.c_in, d.c_out, d.kh, d.kw, d.sw, d.dh, d.dw,
                                              d.residual_from != LOP_NO_RESIDUAL);
  }
  find_fused_groups(P);
  if (flags & LOP_FLAG_BATCH_BANDS) {
    if (flags & LOP_FLAG_REUSE) { delete P; return LOP_ERR_INVALID_ARG; }
    if (!all_launches_batchable(P)) { delete P; return LOP_ERR_UNSUPPORTED; }
    P->batched = true;
  }
  size_scratch(P);
  size_workspace(P);
  if (!(flags & LOP_FLAG_PLAN_ONLY)) {
    rc = setup_device(P);
    if (rc != LOP_OK) { lop_plan_destroy(P); return rc; }
    P->ready = true;
  }
  *out_plan = P;
  return LOP_OK;
}

int lop_plan_rowwise(const lop_rowwise_t* layers, int n_layers, int m, int k, int dtype, int n_bands,
                     unsigned flags, lop_plan_t** out_plan) {
  if (!out_plan) return LOP_ERR_INVALID_ARG;
  *out_plan = nullptr;
  if (!layers || n_layers < 1 || m < 1 || k < 1) return LOP_ERR_INVALID_ARG;
  // a matrix row is a pixel of an m x 1 image with k channels; the product is a 1x1 conv
  std::vector<lop_layer_t> conv((size_t)n_layers);
  for (int l = 0; l < n_layers; ++l) {
    const lop_rowwise_t& r = layers[l];
    lop_layer_t& c = conv[l];
    c.op = LOP_CONV2D;
    c.c_in = r.k; c.c_out = r.n;
    c.kh = c.kw = c.sh = c.sw = c.dh = c.dw = 1;
    c.ph = c.pw = 0;
    c.act = r.act;
    c.input_from = r.input_from;
    c.residual_from = r.residual_from;
    c.weight = r.weight;
    c.bias = r.bias;
  }
  const lop_tensor_desc_t in{1, k, m, 1, dtype};
  return lop_plan(conv.data(), n_layers, &in, n_bands, flags, out_plan);
}

void lop_plan_destroy(lop_plan_t* P) {
  if (!P) return;
  if (P->ready || P->device >= 0) {
    // Everything below belongs to the plan's device, and work that uses the plan's memory may
    // sit on streams the plan does not own (a caller's compute or copy stream, which may not
    // exist any more, so it is not touched through its handle): wait for the whole device.
    int cur = -1;
    if (hipGetDevice(&cur) == hipSuccess && cur != P->device && P->device >= 0) (void)hipSetDevice(P->device);
    (void)hipDeviceSynchronize();
  }
  for (void* w : P->d_w) if (w) (void)lop::dev_free(w);
  for (void* w : P->d_wd) if (w) (void)lop::dev_free(w);
  for (void* w : P->d_wd16) if (w) (void)lop::dev_free(w);
  for (void* w : P->d_wstem) if (w) (void)lop::dev_free(w);
  for (float* b : P->d_bias) if (b) (void)lop::dev_free(b);
  for (auto* v : {&P->ev_done, &P->ev_copied, &P->ev_c0, &P->ev_c1, &P->ev_d0, &P->ev_d1})
    for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
  for (auto& g : P->graphs) (void)hipGraphExecDestroy(g.exec);
  for (hipEvent_t e : {P->ev_fork, P->ev_t0, P->ev_t1, P->ev_copy_tail}) if (e) (void)hipEventDestroy(e);
  for (Lane& L : P->lanes) {
    if (L.arena) (void)lop::dev_free(L.arena);
    if (L.conv_ws) (void)lop::dev_free(L.conv_ws);
    if (L.ev_join) (void)hipEventDestroy(L.ev_join);
    if (L.stream) (void)hipStreamDestroy(L.stream);
    if (L.copy) (void)hipStreamDestroy(L.copy);
  }
  if (P->s_main) (void)hipStreamDestroy(P->s_main);
  if (P->s_copy) (void)hipStreamDestroy(P->s_copy);
  delete P;
}

int lop_plan_out_desc(const lop_plan_t* P, lop_tensor_desc_t* out) {
  if (!P || !out) return LOP_ERR_INVALID_ARG;
  return lop_plan_layer_desc(P, P->t.n_layers() - 1, out);
}

int lop_plan_layer_desc(const lop_plan_t* P, int layer, lop_tensor_desc_t* out) {
  if (!P || !out) return LOP_ERR_INVALID_ARG;
  if (layer < 0 || layer >= P->t.n_layers()) return LOP_ERR_BAND_RANGE;
  const lop::LayerInfo& L = P->t.layers[layer];
  *out = {L.n, L.d.c_out, L.h_out, L.w_out, P->t.in.dtype};
  return LOP_OK;
}

int lop_plan_n_bands(const lop_plan_t* P) { return P ? P->t.n_bands : LOP_ERR_INVALID_ARG; }
int lop_plan_n_layers(const lop_plan_t* P) { return P ? P->t.n_layers() : LOP_ERR_INVALID_ARG; }

int lop_plan_band_layer_rows(const lop_plan_t* P, int band, int layer, lop_rows_t* rows) {
  if (!P || !rows) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands || layer < -1 || layer >= P->t.n_layers())
    return LOP_ERR_BAND_RANGE;
  lop_rows_t r = P->t.bands[band].need[layer + 1];
  if (r.hi <= r.lo) r = {0, 0};
  *rows = r;
  return LOP_OK;
}

int lop_plan_band_out_rows(const lop_plan_t* P, int band, lop_rows_t* rows) {
  if (!P || !rows) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands) return LOP_ERR_BAND_RANGE;
  *rows = P->t.bands[band].need[P->t.n_layers()];  // split intervals keep lo == hi when empty
  return LOP_OK;
}

int lop_plan_band_compute_rows(const lop_plan_t* P, int band, int layer, lop_rows_t* rows) {
  if (!P || !rows) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands || layer < 0 || layer >= P->t.n_layers())
    return LOP_ERR_BAND_RANGE;
  lop_rows_t r = P->t.bands[band].compute[layer];
  if (r.hi <= r.lo) r = {0, 0};
  *rows = r;
  return LOP_OK;
}

int lop_plan_band_in_rows(const lop_plan_t* P, int band, lop_rows_t* rows) {
  return lop_plan_band_layer_rows(P, band, -1, rows);
}

int lop_plan_stats(const lop_plan_t* P, double* useful, double* executed, size_t* scratch) {
  if (!P) return LOP_ERR_INVALID_ARG;
  double u = 0, e = 0;
  for (int l = 0; l < P->t.n_layers(); ++l) {
    u += P->t.layer_flop(l, P->t.layers[l].h_out);
    for (int b = 0; b < P->t.n_bands; ++b) {
      double f = 0.0, by = 0.0;
      if (P->flags & LOP_FLAG_PLAN_ONLY) {  // no kernels are chosen, so no launches are fused
        const lop_rows_t r = P->t.bands[b].compute[l];
        if (r.hi > r.lo) f = P->t.layer_flop(l, r.hi - r.lo);
      } else {
        launch_work(P, b, l, &f, &by);
      }
      e += f;
    }
  }
  if (useful) *useful = u;
  if (executed) *executed = e;
  if (scratch) *scratch = align_up(P->arena_bytes, 256) + P->conv_ws_bytes;
  return LOP_OK;
}

int lop_plan_layer_work(const lop_plan_t* P, int band, int layer, double* flop, double* bytes) {
  if (!P) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands || layer < 0 || layer >= P->t.n_layers())
    return LOP_ERR_BAND_RANGE;
  double f = 0.0, by = 0.0;
  if (P->flags & LOP_FLAG_PLAN_ONLY) {  // no kernels are chosen, so no launches are fused
    const lop_rows_t r = P->t.bands[band].compute[layer];
    f = r.hi > r.lo ? P->t.layer_flop(layer, r.hi - r.lo) : 0.0;
    by = P->t.layer_bytes(band, layer);
  } else {
    launch_work(P, band, layer, &f, &by);
  }
  if (flop) *flop = f;
  if (bytes) *bytes = by;
  return LOP_OK;
}

// The kernels move 16-byte vectors: tensors start on a 16-byte boundary.
static bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

int lop_run_band(lop_plan_t* P, int band, const void* d_in, void* d_out, void* h_out,
                 void* compute_stream, void* copy_stream) {
  if (!P || !d_in || !d_out) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_in) || misaligned(d_out) || misaligned(h_out)) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands) return LOP_ERR_BAND_RANGE;
  if (!P->ready) return LOP_ERR_NOT_READY;
  if (band_empty(P, band)) return LOP_OK;
  if (h_out && !(P->flags & LOP_FLAG_NO_D2H) && !device_view_of_host(P, h_out)) return LOP_ERR_INVALID_ARG;
  hipStream_t cs = compute_stream ? (hipStream_t)compute_stream : P->lane_of(band).stream;
  hipStream_t ds = copy_stream ? (hipStream_t)copy_stream : P->s_copy;
  if (compute_stream) P->last_user_stream = cs;
  return enqueue_band(P, band, d_in, d_out, h_out, cs, ds, false);
}

int lop_run_chain(lop_plan_t* P, const void* d_in, void* d_out, void* h_out, void* compute_stream,
                  lop_timing_t* timing) {
  if (!P || !d_in || !d_out) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_in) || misaligned(d_out) || misaligned(h_out)) return LOP_ERR_INVALID_ARG;
  if (!P->ready) return LOP_ERR_NOT_READY;
  hipStream_t ms = compute_stream ? (hipStream_t)compute_stream : P->s_main;
  if (compute_stream) P->last_user_stream = ms;
  const int nb = P->t.n_bands;
  const bool copy = h_out && !(P->flags & LOP_FLAG_NO_D2H);
  if (copy && !device_view_of_host(P, h_out)) return LOP_ERR_INVALID_ARG;  // not pinned host memory
  if (timing) {
    int rc = ensure_timing_events(P);
    if (rc != LOP_OK) return rc;
    rc = lop_synchronize(P);
    if (rc != LOP_OK) return rc;
  }
  const auto t0 = std::chrono::steady_clock::now();
  if (P->copy_lane && copy && !compute_stream && !timing) {
    // Compute lanes run free, as below; every band's copy goes to the copy lane.
    for (int b = 0; b < nb; ++b) {
      if (band_empty(P, b)) continue;
      int rc = enqueue_band_with_copy_lane(P, b, d_in, d_out, h_out, P->lane_of(b).stream);
      if (rc != LOP_OK) return rc;
    }
    return LOP_OK;
  }
  if (P->t.reuse || P->batched) {
    // the whole chain runs on one lane; chains of consecutive calls rotate over the lanes
    // and overlap unless the caller's stream orders them
    P->cur_lane = P->next_lane;
    P->next_lane = (P->next_lane + 1) % P->n_lanes();
    Lane& L = P->lanes[P->cur_lane];
    if (compute_stream) {
      LOP_HIP(hipEventRecord(P->ev_fork, ms));
      LOP_HIP(hipStreamWaitEvent(L.stream, P->ev_fork, 0));
    }
    if (timing) LOP_HIP(hipEventRecord(P->ev_t0, L.stream));
    int rc = ((P->flags & LOP_FLAG_GRAPH) && !timing)
                 ? launch_graph(P, d_in, d_out, h_out, L.stream)
                 : P->batched ? enqueue_chain_batched(P, d_in, d_out, h_out, timing != nullptr, false)
                              : enqueue_chain_reuse(P, d_in, d_out, h_out, timing != nullptr, false);
    if (rc != LOP_OK) return rc;
    if (timing) LOP_HIP(hipEventRecord(P->ev_t1, L.stream));
    if (compute_stream) {
      LOP_HIP(hipEventRecord(L.ev_join, L.stream));
      LOP_HIP(hipStreamWaitEvent(ms, L.ev_join, 0));
    }
  } else {
    if (!compute_stream && !timing && P->n_lanes() > 1) {
      // No stream of the caller's to order against: every lane takes its bands of this chain
      // behind whatever it still has of earlier chains and nothing joins them, so the lanes
      // drift apart by as much as their bands differ in work and consecutive chains overlap
      // (band b of the next chain starts while slower bands of this one still run). The
      // chain is complete after lop_synchronize.
      for (int k = 0; k < P->n_lanes(); ++k) {
        int rc = (P->flags & LOP_FLAG_GRAPH) ? launch_graph(P, d_in, d_out, h_out, P->lanes[k].stream, k)
                                             : enqueue_lane(P, k, d_in, d_out, h_out, false);
        if (rc != LOP_OK) return rc;
      }
      return LOP_OK;
    }
    if ((P->flags & LOP_FLAG_GRAPH) && !timing) return launch_graph(P, d_in, d_out, h_out, ms);
    if (timing) LOP_HIP(hipEventRecord(P->ev_t0, ms));
    int rc = enqueue_chain(P, d_in, d_out, h_out, ms, timing != nullptr, false);
    if (rc != LOP_OK) return rc;
    if (timing) LOP_HIP(hipEventRecord(P->ev_t1, ms));
  }
  if (!timing) return LOP_OK;
  int rc = lop_synchronize(P);
  if (rc != LOP_OK) return rc;
  const auto t1 = std::chrono::steady_clock::now();
  std::memset(timing, 0, sizeof(*timing));
  timing->n_bands = nb;
  timing->wall_ms = std::chrono::duration<float, std::milli>(t1 - t0).count();
  for (int b = 0; b < nb; ++b) {
    if (band_empty(P, b)) continue;
    LOP_HIP(hipEventElapsedTime(&timing->band_compute_ms[b], P->ev_c0[b], P->ev_c1[b]));
    if (copy) {
      LOP_HIP(hipEventElapsedTime(&timing->band_copy_ms[b], P->ev_d0[b], P->ev_d1[b]));
      timing->copy_ms += timing->band_copy_ms[b];
    }
    LOP_HIP(hipEventElapsedTime(&timing->band_ready_ms[b], P->ev_t0, copy ? P->ev_d1[b] : P->ev_c1[b]));
  }
  LOP_HIP(hipEventElapsedTime(&timing->compute_ms, P->ev_t0, P->ev_t1));
  return LOP_OK;
}

int lop_run_chain_static(lop_plan_t* P, const void* d_in, void* d_out, void* stream) {
  if (!P || !d_in || !d_out) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_in) || misaligned(d_out)) return LOP_ERR_INVALID_ARG;
  if (!P->ready) return LOP_ERR_NOT_READY;
  const size_t arena = align_up(P->arena_bytes, 256);
  if (arena + P->conv_ws_bytes > (size_t)LOP_STATIC_SCRATCH_BYTES) return LOP_ERR_TOO_LARGE;
  unsigned char* const base = (unsigned char*)static_scratch_of(P->device);
  if (!base) return LOP_ERR_NOT_READY;
  // Nothing in the array has to start at zero: a band's slabs are written by the layer that
  // produces them before any layer reads them, and a launch's partial sums by its slices
  // before its finish kernel adds them, so the contents left by the last call do not matter.
  P->arena_override = base;
  P->ws_override = P->conv_ws_bytes ? base + arena : nullptr;
  int rc = LOP_OK;
  for (int b = 0; b < P->t.n_bands && rc == LOP_OK; ++b)
    if (!band_empty(P, b)) rc = enqueue_band_kernels(P, b, d_in, d_out, (hipStream_t)stream);
  P->arena_override = nullptr;
  P->ws_override = nullptr;
  return rc;
}

int lop_synchronize(lop_plan_t* P) {
  if (!P) return LOP_ERR_INVALID_ARG;
  if (!P->ready) return LOP_ERR_NOT_READY;
  if (P->last_user_stream) LOP_HIP(hipStreamSynchronize(P->last_user_stream));
  for (Lane& L : P->lanes) {
    LOP_HIP(hipStreamSynchronize(L.stream));
    LOP_HIP(hipStreamSynchronize(L.copy));
  }
  LOP_HIP(hipStreamSynchronize(P->s_main));
  LOP_HIP(hipStreamSynchronize(P->s_copy));
  return LOP_OK;
}

int lop_time_layer(lop_plan_t* P, int band, int layer, const void* d_in, void* d_out, int iters,
                   float* ms_per_launch) {
  if (!P || !d_in || !d_out || !ms_per_launch || iters < 1) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_in) || misaligned(d_out)) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands || layer < 0 || layer >= P->t.n_layers())
    return LOP_ERR_BAND_RANGE;
  if (!P->ready) return LOP_ERR_NOT_READY;
  *ms_per_launch = 0.f;
  const lop_rows_t r = launch_rows(P, band, layer);
  if (r.hi <= r.lo) return LOP_OK;
  int rc = ensure_timing_events(P);
  if (rc != LOP_OK) return rc;
  hipStream_t cs = P->s_main;
  LOP_HIP(launch_layer(P, band, layer, d_in, d_out, cs));  // warm-up
  LOP_HIP(hipEventRecord(P->ev_c0[0], cs));
  for (int i = 0; i < iters; ++i) LOP_HIP(launch_layer(P, band, layer, d_in, d_out, cs));
  LOP_HIP(hipEventRecord(P->ev_c1[0], cs));
  LOP_HIP(hipStreamSynchronize(cs));
  float ms = 0.f;
  LOP_HIP(hipEventElapsedTime(&ms, P->ev_c0[0], P->ev_c1[0]));
  *ms_per_launch = ms / iters;
  return LOP_OK;
}

int lop_plan_layer_kernel(const lop_plan_t* P, int band, int layer, char* name, size_t size,
                          int* k_slices) {
  if (!P || !name || size == 0) return LOP_ERR_INVALID_ARG;
  if (band < 0 || band >= P->t.n_bands || layer < 0 || layer >= P->t.n_layers())
    return LOP_ERR_BAND_RANGE;
  name[0] = 0;
  int slices = 0;
  // (a plan-only plan has uploaded no weights, and which kernel takes a layer depends on the
  // packings that exist: it names none rather than a kernel the ready plan would not launch)
  if (P->flags & LOP_FLAG_PLAN_ONLY) {
  } else if (P->batched) {   // one launch per layer for all bands: named at the first band that takes part
    if (batched_owner(P, layer) == band) slices = describe_layer_batched(P, layer, name, size);
  } else {
    slices = describe_layer_launch(P, band, layer, name, size);
  }
  if (k_slices) *k_slices = slices;
  return LOP_OK;
}

int lop_profile_chain(lop_plan_t* P, const void* d_in, void* d_out, int iters, float* layer_ms,
                      float* finish_ms) {
  if (!P || !d_in || !d_out || !layer_ms || iters < 1) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_in) || misaligned(d_out)) return LOP_ERR_INVALID_ARG;
  if (!P->ready) return LOP_ERR_NOT_READY;
  const int nb = P->t.n_bands, nl = P->t.n_layers();
  int rc = lop_synchronize(P);
  if (rc != LOP_OK) return rc;
  hipStream_t cs = P->s_main;
  // (start, stop) of the operator's kernel and of its finish kernel, attached to the
  // dispatches themselves
  std::vector<hipEvent_t> ev((size_t)nb * nl * 4, nullptr);
  std::vector<int> used((size_t)nb * nl, 0);
  auto run = [&]() -> int {
    for (auto& e : ev) LOP_HIP(hipEventCreate(&e));
    for (int i = 0; i < nb * nl; ++i) {
      layer_ms[i] = 0.f;
      if (finish_ms) finish_ms[i] = 0.f;
    }
    for (int it = 0; it < iters; ++it) {
      for (int b = 0; b < nb; ++b)
        for (int l = 0; l < nl; ++l) {
          const lop_rows_t r = launch_rows(P, b, l);
          if (r.hi <= r.lo) continue;
          if (P->batched && batched_owner(P, l) != b) continue;  // (timed with the band that owns the launch)
          const size_t i = ((size_t)b * nl + l) * 4;
          lop::KernelEvents ke;
          ke.start[0] = ev[i]; ke.stop[0] = ev[i + 1];
          ke.start[1] = ev[i + 2]; ke.stop[1] = ev[i + 3];
          if (P->batched) LOP_HIP(launch_layer_batched(P, l, d_in, d_out, cs, &ke, nullptr, nullptr));
          else LOP_HIP(launch_layer(P, b, l, d_in, d_out, cs, &ke));
          used[b * nl + l] = ke.n;
        }
      LOP_HIP(hipStreamSynchronize(cs));
      for (int b = 0; b < nb; ++b)
        for (int l = 0; l < nl; ++l) {
          const size_t i = ((size_t)b * nl + l) * 4;
          float ms = 0.f, fin = 0.f;
          if (used[b * nl + l] >= 1) LOP_HIP(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
          if (used[b * nl + l] >= 2) LOP_HIP(hipEventElapsedTime(&fin, ev[i + 2], ev[i + 3]));
          layer_ms[b * nl + l] += ms / iters;
          if (finish_ms) finish_ms[b * nl + l] += fin / iters;
        }
    }
    return LOP_OK;
  };
  rc = run();
  for (hipEvent_t e : ev) if (e) (void)hipEventDestroy(e);
  return rc;
}

int lop_copy_chain(lop_plan_t* P, const void* d_out, void* h_out) {
  if (!P || !d_out || !h_out) return LOP_ERR_INVALID_ARG;
  if (misaligned(d_out) || misaligned(h_out)) return LOP_ERR_INVALID_ARG;
  if (!P->ready) return LOP_ERR_NOT_READY;
  if (!device_view_of_host(P, h_out)) return LOP_ERR_INVALID_ARG;
  for (int b = 0; b < P->t.n_bands; ++b) {
    int rc = enqueue_band_copy(P, b, d_out, h_out, P->s_copy);
    if (rc != LOP_OK) return rc;
  }
  return LOP_OK;
}

const char* lop_strerror(int code) {
  switch (code) {
    case LOP_OK: return "ok";
    case LOP_ERR_INVALID_ARG: return "invalid argument";
    case LOP_ERR_UNSUPPORTED: return "unsupported operator, type or parameter";
    case LOP_ERR_SHAPE: return "shape mismatch";
    case LOP_ERR_BAND_RANGE: return "band or layer index out of range";
    case LOP_ERR_OOM: return "out of memory";
    case LOP_ERR_HIP: return "HIP runtime error";
    case LOP_ERR_NOT_READY: return "plan holds no device state (plan-only)";
    case LOP_ERR_TOO_LARGE: return "the plan needs more scratch than the static array holds";
    default: return "unknown error";
  }
}

int lop_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
