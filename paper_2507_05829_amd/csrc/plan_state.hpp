// State behind a lop_plan_t handle, shared by the sources that implement the C ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <utility>
#include <vector>

#include "kernels.hpp"
#include "lop.h"
#include "plan_tables.hpp"

namespace lop {
// Remembers the HIP error for lop_last_hip_error() and maps it to a lop_status_t.
int hip_fail(hipError_t e);
}  // namespace lop

#define LOP_HIP(call)                                \
  do {                                               \
    hipError_t e_ = (call);                          \
    if (e_ != hipSuccess) return lop::hip_fail(e_);  \
  } while (0)

// One lane = one compute stream with its own scratch; bands are dealt to lanes round
// robin and the lanes run concurrently (bands are independent of one another).
struct Lane {
  hipStream_t stream = nullptr;
  hipStream_t copy = nullptr;  // reuse mode: this lane's copies overlap its next band
  void* arena = nullptr;    // scratch slabs of one band at a time
  void* conv_ws = nullptr;  // split-K partial sums of one launch at a time
  hipEvent_t ev_join = nullptr;
};

struct lop_plan_s {
  lop::Tables t;
  unsigned flags = 0;
  bool ready = false;
  int device = -1;
  std::vector<void*> d_w;      // per layer packed weights (device) or nullptr
  std::vector<void*> d_wd;     // dense conv weights in MFMA operand order, or nullptr
  std::vector<void*> d_wd16;   // ... in the operand order of 16 x 16 tiles, or nullptr
  std::vector<void*> d_wstem;  // ... as fp32 [c_out / 4][k][4] for the first-layer kernel, or nullptr
  // Layers that run as one launch: fuse_head[t] = first layer of the group whose last layer is
  // t (else -1); fused_away[l] = 1 for the layers of a group before its last (no launch, no
  // buffer of their own).
  std::vector<int> fuse_head;
  std::vector<char> fused_away;
  std::vector<float*> d_bias;  // per layer bias (device) or nullptr
  std::vector<int> k_pad;
  std::vector<char> has_wd, has_wd16;  // which of the two operand-order packings a layer gets
  std::vector<char> has_wstem;         // ... and whether it gets the first-layer packing
  size_t conv_ws_bytes = 0;
  size_t arena_bytes = 0;
  std::vector<std::vector<size_t>> slab_off;  // [band][layer] byte offset into a lane's arena
  std::vector<Lane> lanes;
  hipStream_t s_main = nullptr, s_copy = nullptr;
  hipStream_t last_user_stream = nullptr;
  hipEvent_t ev_fork = nullptr;
  std::vector<hipEvent_t> ev_done;                          // per band: kernels finished
  std::vector<hipEvent_t> ev_copied;                        // per band: last copy finished
  std::vector<char> copied_valid;
  std::vector<hipEvent_t> ev_c0, ev_c1, ev_d0, ev_d1;       // timing only (lazy)
  hipEvent_t ev_t0 = nullptr, ev_t1 = nullptr;
  hipEvent_t ev_copy_tail = nullptr;
  struct GraphEntry {
    const void* d_in; void* d_out; void* h_out;
    int lane;
    int band;  // -1: every band of the lane (or chain); else that band's kernels only
    hipGraphExec_t exec;
  };
  std::vector<GraphEntry> graphs;  // LOP_FLAG_GRAPH: one instantiated graph per pointer set
  std::vector<std::pair<void*, void*>> host_views;  // host buffer -> device-side address

  int cur_lane = 0;   // reuse mode: the lane the chain being enqueued runs on
  int next_lane = 0;  // reuse mode: rotates with every lop_run_chain

  // The last lane carries nothing but band copies when the bands' copies are long (see
  // setup_device): the other lanes never wait for a copy, and the copies of equal bands, which
  // would otherwise all fall into the same moments, follow each other on one stream.
  bool copy_lane = false;
  int n_lanes() const { return (int)lanes.size() - (copy_lane ? 1 : 0); }  // lanes that compute
  // Independent bands are dealt to the lanes round robin; in reuse mode a whole chain (all
  // bands, in order) runs on one lane and consecutive chains rotate over the lanes.
  bool batched = false;  // LOP_FLAG_BATCH_BANDS: one launch per layer for all bands, a chain per lane
  int lane_index(int band) const { return t.reuse || batched ? cur_lane : band % n_lanes(); }
  Lane& lane_of(int band) { return lanes[lane_index(band)]; }
  const Lane& lane_of(int band) const { return lanes[lane_index(band)]; }
  // While lop_run_chain_static enqueues, scratch comes from the library's static device array
  // instead of the lanes' allocations.
  void* arena_override = nullptr;
  void* ws_override = nullptr;
  void* arena_of(int band) const {
    if (arena_override) return arena_override;
    return lanes.empty() ? nullptr : lane_of(band).arena;
  }
  void* ws_of(int band) const {
    if (ws_override) return ws_override;
    return lanes.empty() ? nullptr : lane_of(band).conv_ws;
  }
};

namespace lop {
// Operator parameters of layer l without any slab (x.c and y.c are set; res.ptr is a non-null
// marker when the layer adds a residual): what the kernel selection looks at, and the base
// of a launch once its slabs and output rows are filled in.
OpLaunch describe_layer(const lop_plan_s* P, int l);
}  // namespace lop
