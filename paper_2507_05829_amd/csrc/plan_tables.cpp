// Shape inference, band split and backward halo propagation (host, integers only).
//
// A windowed local operator's output row oh reads input rows oh*s - p + a*d, a in [0,k)
// (Intra-DP Sec. IV-A: the input block of a block-wise operator follows from kernel
// size, padding and dilation). An interval [lo,hi) of output rows therefore needs the
// input interval [lo*s - p, (hi-1)*s - p + d*(k-1) + 1), clamped to the image. A tensor
// with several consumers (shortcut branch, residual read) is needed on the hull of
// their intervals so that one launch covers one contiguous interval (Sec. IV-C,
// Computational Efficiency); rows two bands both need are computed by both (local
// operation replication, Sec. IV-C), which makes the bands independent.
#include "plan_tables.hpp"

#include <algorithm>

namespace lop {

int out_size(int in, int k, int s, int p, int d) {
  const long span = (long)in + 2L * p - (long)d * (k - 1) - 1;
  if (span < 0) return 0;
  return (int)(span / s) + 1;
}

void split_rows(int h, int n, std::vector<lop_rows_t>& out) {
  out.resize(n);
  const int base = h / n, extra = h % n;
  int lo = 0;
  for (int b = 0; b < n; ++b) {
    const int hi = lo + base + (b < extra ? 1 : 0);
    out[b] = {lo, hi};
    lo = hi;
  }
}

static inline bool empty(const lop_rows_t& r) { return r.hi <= r.lo; }

static inline void hull_into(lop_rows_t& dst, const lop_rows_t& src) {
  if (empty(src)) return;
  if (empty(dst)) { dst = src; return; }
  dst.lo = std::min(dst.lo, src.lo);
  dst.hi = std::max(dst.hi, src.hi);
}

double Tables::layer_flop(int l, int rows) const {
  const LayerInfo& L = layers[l];
  const double px = (double)L.n * rows * L.w_out;
  switch (L.d.op) {
    case LOP_CONV2D:
    case LOP_DWCONV2D:  // padding taps are counted: an implicit GEMM multiplies them too
      return 2.0 * px * L.d.c_out * (L.d.c_in / L.groups) * L.d.kh * L.d.kw;
    case LOP_MAXPOOL2D:
      return px * L.d.c_out * L.d.kh * L.d.kw;
    default:
      return px * L.d.c_out;
  }
}

double Tables::layer_bytes(int band, int l) const {
  const LayerInfo& L = layers[l];
  const BandRows& B = bands[band];
  const lop_rows_t out = B.compute[l];
  if (empty(out)) return 0.0;
  const lop_rows_t rd = B.reads[l];
  const double e = (double)esz();
  double bytes = e * L.n * ((double)(rd.hi - rd.lo) * L.w_in * L.d.c_in +
                            (double)(out.hi - out.lo) * L.w_out * L.d.c_out);
  if (L.d.residual_from != LOP_NO_RESIDUAL)
    bytes += e * L.n * (double)(out.hi - out.lo) * L.w_out * L.d.c_out;
  if (L.d.op == LOP_CONV2D || L.d.op == LOP_DWCONV2D)
    bytes += e * (double)L.d.c_out * (L.d.c_in / L.groups) * L.d.kh * L.d.kw;
  return bytes;
}

static lop_rows_t reads_of(const LayerInfo& L, lop_rows_t o) {
  lop_rows_t src{0, 0};
  if (empty(o)) return src;
  src.lo = std::max(o.lo * L.d.sh - L.d.ph, 0);
  src.hi = std::min((o.hi - 1) * L.d.sh - L.d.ph + L.d.dh * (L.d.kh - 1) + 1, L.h_in);
  if (src.hi < src.lo) src.hi = src.lo;
  return src;
}

int build_tables(const lop_layer_t* layers, int n_layers, const lop_tensor_desc_t* in,
                 int n_bands, bool reuse, Tables& t) {
  if (!layers || !in || n_layers < 1) return LOP_ERR_INVALID_ARG;
  if (n_bands < 1 || n_bands > LOP_MAX_BANDS) return LOP_ERR_INVALID_ARG;
  if (in->n < 1 || in->c < 1 || in->h < 1 || in->w < 1) return LOP_ERR_INVALID_ARG;
  if (in->dtype != LOP_F32 && in->dtype != LOP_BF16) return LOP_ERR_UNSUPPORTED;
  t.in = *in;
  t.n_bands = n_bands;
  t.reuse = reuse;
  t.layers.assign(n_layers, LayerInfo{});

  // ---- forward: shapes
  for (int i = 0; i < n_layers; ++i) {
    LayerInfo& L = t.layers[i];
    L.d = layers[i];
    const lop_layer_t& d = L.d;
    if (d.op < LOP_CONV2D || d.op > LOP_ELTWISE) return LOP_ERR_UNSUPPORTED;
    if (d.act < LOP_ACT_NONE || d.act > LOP_ACT_RELU6) return LOP_ERR_UNSUPPORTED;
    if (d.input_from < LOP_INPUT || d.input_from >= i) return LOP_ERR_INVALID_ARG;
    if (d.residual_from < LOP_NO_RESIDUAL || d.residual_from >= i) return LOP_ERR_INVALID_ARG;
    if (d.c_in < 1 || d.c_out < 1) return LOP_ERR_INVALID_ARG;
    const int src = d.input_from;
    const int c_src = src < 0 ? in->c : t.layers[src].d.c_out;
    L.n = in->n;
    L.h_in = t.tensor_h(src);
    L.w_in = src < 0 ? in->w : t.layers[src].w_out;
    if (d.c_in != c_src) return LOP_ERR_SHAPE;
    if (d.op != LOP_CONV2D && d.c_out != d.c_in) return LOP_ERR_SHAPE;
    L.groups = d.op == LOP_DWCONV2D ? d.c_in : 1;
    if (d.op == LOP_ELTWISE) {
      L.d.kh = L.d.kw = L.d.sh = L.d.sw = L.d.dh = L.d.dw = 1;
      L.d.ph = L.d.pw = 0;
      L.h_out = L.h_in;
      L.w_out = L.w_in;
    } else {
      if (d.kh < 1 || d.kw < 1 || d.sh < 1 || d.sw < 1 || d.ph < 0 || d.pw < 0 || d.dh < 1 ||
          d.dw < 1)
        return LOP_ERR_INVALID_ARG;
      L.h_out = out_size(L.h_in, d.kh, d.sh, d.ph, d.dh);
      L.w_out = out_size(L.w_in, d.kw, d.sw, d.pw, d.dw);
      if (L.h_out < 1 || L.w_out < 1) return LOP_ERR_SHAPE;
    }
    if (d.op == LOP_MAXPOOL2D) {
      if (d.bias || d.residual_from != LOP_NO_RESIDUAL || d.act != LOP_ACT_NONE)
        return LOP_ERR_INVALID_ARG;
      // a window that lies wholly in the padding has no defined maximum
      if (d.ph >= d.kh || d.pw >= d.kw || d.dh != 1 || d.dw != 1) return LOP_ERR_UNSUPPORTED;
    }
    if (d.residual_from != LOP_NO_RESIDUAL) {
      const int r = d.residual_from;
      const int rc = r < 0 ? in->c : t.layers[r].d.c_out;
      const int rh = t.tensor_h(r);
      const int rw = r < 0 ? in->w : t.layers[r].w_out;
      if (rc != d.c_out || rh != L.h_out || rw != L.w_out) return LOP_ERR_SHAPE;
    }
  }

  // ---- bands on the last layer's rows, then backwards
  std::vector<lop_rows_t> out_rows;
  split_rows(t.layers.back().h_out, n_bands, out_rows);
  t.bands.assign(n_bands, BandRows{});
  for (int b = 0; b < n_bands; ++b) {
    BandRows& B = t.bands[b];
    B.need.assign(n_layers + 1, lop_rows_t{0, 0});
    B.reads.assign(n_layers, lop_rows_t{0, 0});
    B.need[n_layers] = out_rows[b];
    for (int i = n_layers - 1; i >= 0; --i) {
      const LayerInfo& L = t.layers[i];
      const lop_rows_t o = B.need[i + 1];
      if (empty(o)) continue;
      const lop_rows_t src = reads_of(L, o);
      hull_into(B.need[L.d.input_from + 1], src);
      if (L.d.residual_from != LOP_NO_RESIDUAL) hull_into(B.need[L.d.residual_from + 1], o);
    }
  }
  // ---- what each band's launches produce. The needed intervals move monotonically down
  // the image with the band index, so "rows some earlier band produced" is everything
  // below the highest `hi` seen so far; rows of need[] below that mark are already there.
  std::vector<int> done_hi(n_layers, 0);
  for (int b = 0; b < n_bands; ++b) {
    BandRows& B = t.bands[b];
    B.compute.assign(n_layers, lop_rows_t{0, 0});
    for (int i = 0; i < n_layers; ++i) {
      lop_rows_t c = B.need[i + 1];
      if (empty(c)) continue;
      if (reuse) {
        c.lo = std::max(c.lo, done_hi[i]);
        if (c.hi <= c.lo) { c = {0, 0}; }
        done_hi[i] = std::max(done_hi[i], B.need[i + 1].hi);
      }
      B.compute[i] = c;
      B.reads[i] = reads_of(t.layers[i], c);
    }
  }
  return LOP_OK;
}

}  // namespace lop
