// Host-side integer planning for a banded chain of local operators.
// Pure arithmetic: no HIP calls, usable without a GPU.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "lop.h"

namespace lop {

struct LayerInfo {
  lop_layer_t d;        // caller's descriptor (weight/bias pointers are not kept valid)
  int n = 0;            // batch
  int h_in = 0, w_in = 0;
  int h_out = 0, w_out = 0;
  int groups = 1;
};

// Row intervals of one band. need[0] is the chain input, need[l + 1] is layer l's output.
struct BandRows {
  std::vector<lop_rows_t> need;
  // compute[l]: rows of layer l's output this band's launch produces. Independent bands:
  // all of need[l + 1]. Reuse mode: only the rows no earlier band has produced.
  std::vector<lop_rows_t> compute;
  // reads[l]: rows of layer l's *input* tensor that the launch touches (the producer's
  // slab may be larger because of other consumers).
  std::vector<lop_rows_t> reads;
};

struct Tables {
  lop_tensor_desc_t in{};
  int n_bands = 0;
  bool reuse = false;
  std::vector<LayerInfo> layers;
  std::vector<BandRows> bands;

  int n_layers() const { return (int)layers.size(); }
  size_t esz() const { return in.dtype == LOP_BF16 ? 2 : 4; }
  // Elements per row (all images excluded): W * C of tensor t (t = -1: chain input).
  int64_t row_elems(int t) const {
    return t < 0 ? (int64_t)in.w * in.c : (int64_t)layers[t].w_out * layers[t].d.c_out;
  }
  int tensor_h(int t) const { return t < 0 ? in.h : layers[t].h_out; }
  double layer_flop(int l, int rows) const;
  double layer_bytes(int band, int l) const;
};

// Output size of a windowed operator, floor mode; <= 0 when the window does not fit.
int out_size(int in, int k, int s, int p, int d);

// Split [0, h) into n intervals: the first h % n are one longer; later ones may be empty.
void split_rows(int h, int n, std::vector<lop_rows_t>& out);

// Validate the chain and fill shapes and per-band row intervals. Returns a lop_status_t.
// reuse: bands run in order and share per-layer buffers, so a band only computes the rows
// of each layer that bands before it have not produced (no halo recompute).
int build_tables(const lop_layer_t* layers, int n_layers, const lop_tensor_desc_t* in,
                 int n_bands, bool reuse, Tables& t);

}  // namespace lop
