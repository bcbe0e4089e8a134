// Two parties on one GPU executing a schedule of local operations (Sec. IV-D, Alg. 1 client
// and Alg. 2 server): each party is a stream with buffers of its own, the link between them a
// pair of streams (one per direction) whose copies are followed by a timed wait that stands
// for latency + bytes / bandwidth. An emulation for studying schedules, not the hot path.
#include <hip/hip_runtime.h>

#include <cstdint>

#include <algorithm>
#include <vector>

#include "devmem.hpp"
#include "plan_state.hpp"

namespace {

constexpr double kMaxDelaySeconds = 2.0;  // longest single emulated wait the call accepts

// Holds a stream for `ticks` of the constant-rate wall clock. Every lane leaves the loop when
// the clock says so, and after a number of polls that is proportional to the wait even if the
// clock did not move (a poll sleeps about a microsecond, i.e. about 100 ticks).
__global__ void delay_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  const long long max_polls = ticks / 16 + 1024;
  for (long long i = 0; i < max_polls; ++i) {
    if (wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(32);
  }
}

struct Piece { int lo, hi; };

// need minus the union of held, as sorted disjoint pieces
std::vector<Piece> subtract(Piece need, const std::vector<Piece>& held) {
  std::vector<Piece> out;
  if (need.hi > need.lo) out.push_back(need);
  for (const Piece& h : held) {
    if (h.hi <= h.lo) continue;
    std::vector<Piece> nxt;
    for (const Piece& p : out) {
      if (h.hi <= p.lo || h.lo >= p.hi) { nxt.push_back(p); continue; }
      if (p.lo < h.lo) nxt.push_back(Piece{p.lo, h.lo});
      if (h.hi < p.hi) nxt.push_back(Piece{h.hi, p.hi});
    }
    out.swap(nxt);
  }
  return out;
}

struct Party {
  hipStream_t compute = nullptr;
  hipStream_t link_in = nullptr;           // carries rows to this party
  std::vector<void*> buf;                  // [tensor + 1]; full height, rows at their position
  std::vector<std::vector<Piece>> held;    // [tensor + 1]: rows computed or received
  std::vector<hipEvent_t> done;            // [tensor + 1]: this party's rows of it are computed
  std::vector<std::vector<hipEvent_t>> wait_for;  // [layer]: arrivals its launch depends on
  void* arena = nullptr;
  void* ws = nullptr;
};

// Everything the call creates, released on every way out.
struct Session {
  Party party[2];  // 0 = M (client), 1 = R (server)
  std::vector<hipEvent_t> events;
  hipEvent_t t0 = nullptr, t1 = nullptr;
  ~Session() {
    // wait for all four streams, then release in the reverse order of dependence: events
    // (recorded on, and waited for by, the streams) before the streams, buffers last
    for (Party& p : party) {
      if (p.compute) (void)hipStreamSynchronize(p.compute);
      if (p.link_in) (void)hipStreamSynchronize(p.link_in);
    }
    for (hipEvent_t e : events) (void)hipEventDestroy(e);
    if (t0) (void)hipEventDestroy(t0);
    if (t1) (void)hipEventDestroy(t1);
    for (Party& p : party) {
      if (p.compute) (void)hipStreamDestroy(p.compute);
      if (p.link_in) (void)hipStreamDestroy(p.link_in);
    }
    for (Party& p : party) {
      if (p.arena) (void)lop::dev_free(p.arena);
      if (p.ws) (void)lop::dev_free(p.ws);
    }
  }
  hipError_t new_event(hipEvent_t* e) {
    const hipError_t rc = hipEventCreateWithFlags(e, hipEventDisableTiming);
    if (rc == hipSuccess) events.push_back(*e);
    return rc;
  }
};

inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

extern "C" int lop_run_two_party(lop_plan_t* P, const void* d_in, void* d_out, const lop_loss_alloc_t* sched,
                                 int n_sched, const lop_loss_layer_t* costs, double bandwidth,
                                 double latency, lop_two_party_stats_t* stats) {
  if (!P || !d_in || !d_out || !sched) return LOP_ERR_INVALID_ARG;
  if ((((uintptr_t)d_in | (uintptr_t)d_out) & 15u) != 0) return LOP_ERR_INVALID_ARG;   // 16-byte vectors
  const lop::Tables& t = P->t;
  const int nl = t.n_layers();
  if (n_sched != nl || !(bandwidth > 0.0) || latency < 0.0) return LOP_ERR_INVALID_ARG;
  // partitioning and batching constraints (Sec. IV-C): two intervals whose union is OP(v)
  for (int v = 0; v < nl; ++v) {
    const int h = t.layers[v].h_out;
    const lop_loss_alloc_t& a = sched[v];
    if (a.m_lo < 0 || a.m_lo > a.m_hi || a.m_hi > h || a.r_lo < 0 || a.r_lo > a.r_hi || a.r_hi > h)
      return LOP_ERR_BAND_RANGE;
    std::vector<Piece> rest = subtract(Piece{0, h}, {Piece{a.m_lo, a.m_hi}, Piece{a.r_lo, a.r_hi}});
    if (!rest.empty()) return LOP_ERR_BAND_RANGE;
  }
  if (!P->ready) return LOP_ERR_NOT_READY;

  const size_t esz = t.esz();
  auto rows_of = [&](int u) { return t.tensor_h(u); };
  auto row_bytes = [&](int u) { return (size_t)t.row_elems(u) * esz; };  // one row of one image
  auto xrows = [&](int v, int d) {
    return d == 0 ? Piece{sched[v].m_lo, sched[v].m_hi} : Piece{sched[v].r_lo, sched[v].r_hi};
  };
  auto cost_seconds = [&](int v, int d, int rows) {
    if (!costs || rows <= 0) return 0.0;
    return d == 0 ? costs[v].cm_fixed + costs[v].cm_row * rows : costs[v].cr_fixed + costs[v].cr_row * rows;
  };
  // every emulated wait has to be short enough for the bounded delay kernel
  for (int v = 0; v < nl; ++v)
    for (int d = 0; d < 2; ++d) {
      const Piece x = xrows(v, d);
      const double c = cost_seconds(v, d, x.hi - x.lo);
      if (!(c >= 0.0) || c > kMaxDelaySeconds) return LOP_ERR_INVALID_ARG;
    }

  int device = 0, clock_khz = 0;
  LOP_HIP(hipGetDevice(&device));
  LOP_HIP(hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, device));
  if (clock_khz <= 0) return LOP_ERR_UNSUPPORTED;
  auto ticks_of = [&](double seconds) { return (long long)(seconds * 1e3 * clock_khz + 0.5); };

  Session S;
  // ---- buffers: the client's input and result are the caller's, everything else is per party
  std::vector<size_t> off(nl + 1, 0);
  size_t total = 0;
  for (int u = -1; u < nl; ++u) {
    off[u + 1] = total;
    total += align256((size_t)t.in.n * rows_of(u) * row_bytes(u));
  }
  size_t ws_bytes = 0;
  std::vector<lop::OpLaunch> launch[2];
  for (int d = 0; d < 2; ++d) {
    Party& p = S.party[d];
    LOP_HIP(lop::dev_alloc(&p.arena, total));
    p.buf.resize(nl + 1);
    for (int u = -1; u < nl; ++u) p.buf[u + 1] = (char*)p.arena + off[u + 1];
    if (d == 0) {
      p.buf[0] = const_cast<void*>(d_in);
      p.buf[nl] = d_out;
    }
    p.held.assign(nl + 1, {});
    p.done.assign(nl + 1, nullptr);
    p.wait_for.assign(nl + 1, {});
    for (auto& e : p.done) LOP_HIP(S.new_event(&e));
    LOP_HIP(hipStreamCreateWithFlags(&p.compute, hipStreamNonBlocking));
    LOP_HIP(hipStreamCreateWithFlags(&p.link_in, hipStreamNonBlocking));
    // one launch per (party, layer): the layer's operator on the party's interval, slabs at full height
    launch[d].resize(nl);
    for (int v = 0; v < nl; ++v) {
      const lop_layer_t& L = t.layers[v].d;
      lop::OpLaunch o = lop::describe_layer(P, v);
      auto slab = [&](int u) {
        lop::Slab s;
        s.ptr = p.buf[u + 1];
        s.n = t.in.n; s.h = rows_of(u);
        s.w = u < 0 ? t.in.w : t.layers[u].w_out;
        s.c = u < 0 ? t.in.c : t.layers[u].d.c_out;
        s.row0 = 0; s.rows = s.h;
        return s;
      };
      o.x = slab(L.input_from);
      o.y = slab(v);
      if (L.residual_from != LOP_NO_RESIDUAL) o.res = slab(L.residual_from);
      const Piece x = xrows(v, d);
      o.out_lo = x.lo; o.out_hi = x.hi;
      launch[d][v] = o;
      if (o.op == LOP_CONV2D && x.hi > x.lo && !lop::pointwise_applies(o))
        ws_bytes = std::max(ws_bytes, lop::conv_workspace_bytes(o));
    }
  }
  for (int d = 0; d < 2; ++d) {
    if (ws_bytes) LOP_HIP(lop::dev_alloc(&S.party[d].ws, ws_bytes));
    for (auto& o : launch[d]) o.ws = S.party[d].ws;
  }
  S.party[0].held[0].push_back(Piece{0, rows_of(-1)});  // the client holds the whole input

  double bytes_to[2] = {0.0, 0.0};
  int transfers = 0;

  // Rows of tensor u that the operations `x` of layer v read through the windowed edge
  // (identity: the residual edge and the edge to the result read the same rows).
  auto reads = [&](int v, Piece x, int u, bool identity) {
    if (x.hi <= x.lo) return Piece{0, 0};
    const lop_layer_t& L = t.layers[v].d;
    if (identity || L.op == LOP_ELTWISE) return x;
    const int lo = std::max(x.lo * L.sh - L.ph, 0);
    const int hi = std::min((x.hi - 1) * L.sh - L.ph + L.dh * (L.kh - 1) + 1, rows_of(u));
    return Piece{lo, std::max(lo, hi)};
  };

  // Send / Receive / combine for every edge out of u (Alg. 1 and 2, the loop over edges): the
  // rows party d will read and does not hold travel from its peer on the link into d.
  // dry: only follow who holds what and check that every wait is short enough to emulate.
  auto exchange = [&](int u, bool dry) -> int {
    struct Edge { int v; bool identity; };
    std::vector<Edge> edges;
    for (int v = 0; v < nl; ++v) {
      if (t.layers[v].d.input_from == u) edges.push_back(Edge{v, false});
      if (t.layers[v].d.residual_from == u) edges.push_back(Edge{v, true});
    }
    if (u == nl - 1) edges.push_back(Edge{nl, true});
    const size_t rb = row_bytes(u), pitch = (size_t)rows_of(u) * rb;
    for (const Edge& e : edges)
      for (int d = 0; d < 2; ++d) {
        Party& me = S.party[d];
        Party& peer = S.party[1 - d];
        Piece need;
        if (e.v == nl) need = d == 0 ? Piece{0, rows_of(u)} : Piece{0, 0};  // the result stays on the client
        else need = reads(e.v, xrows(e.v, d), u, e.identity);
        for (const Piece& pc : subtract(need, me.held[u + 1])) {
          if (dry) {
            if (latency + (double)(pc.hi - pc.lo) * rb * t.in.n / bandwidth > kMaxDelaySeconds)
              return LOP_ERR_INVALID_ARG;
            me.held[u + 1].push_back(pc);
            continue;
          }
          LOP_HIP(hipStreamWaitEvent(me.link_in, peer.done[u + 1], 0));
          LOP_HIP(hipMemcpy2DAsync((char*)me.buf[u + 1] + (size_t)pc.lo * rb, pitch,
                                   (const char*)peer.buf[u + 1] + (size_t)pc.lo * rb, pitch,
                                   (size_t)(pc.hi - pc.lo) * rb, t.in.n, hipMemcpyDeviceToDevice,
                                   me.link_in));
          const double nbytes = (double)(pc.hi - pc.lo) * rb * t.in.n;
          hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, me.link_in,
                             ticks_of(latency + nbytes / bandwidth));
          LOP_HIP(hipGetLastError());
          hipEvent_t arrived;
          LOP_HIP(S.new_event(&arrived));
          LOP_HIP(hipEventRecord(arrived, me.link_in));
          me.wait_for[e.v].push_back(arrived);
          me.held[u + 1].push_back(pc);
          bytes_to[d] += nbytes;
          ++transfers;
        }
      }
    return LOP_OK;
  };

  // first pass without the GPU: the messages this schedule causes, checked against the limit
  for (int u = -1; u < nl; ++u) {
    if (u >= 0)
      for (int d = 0; d < 2; ++d) {
        const Piece x = xrows(u, d);
        if (x.hi > x.lo) S.party[d].held[u + 1].push_back(x);
      }
    const int rc_dry = exchange(u, true);
    if (rc_dry != LOP_OK) return rc_dry;
  }
  for (Party& p : S.party) p.held.assign(nl + 1, {});
  S.party[0].held[0].push_back(Piece{0, rows_of(-1)});

  LOP_HIP(hipEventCreate(&S.t0));
  LOP_HIP(hipEventCreate(&S.t1));
  LOP_HIP(hipDeviceSynchronize());
  LOP_HIP(hipEventRecord(S.t0, S.party[0].compute));
  // the other three streams start when the client does
  LOP_HIP(hipStreamWaitEvent(S.party[1].compute, S.t0, 0));
  LOP_HIP(hipStreamWaitEvent(S.party[0].link_in, S.t0, 0));
  LOP_HIP(hipStreamWaitEvent(S.party[1].link_in, S.t0, 0));
  LOP_HIP(hipEventRecord(S.party[0].done[0], S.party[0].compute));
  LOP_HIP(hipEventRecord(S.party[1].done[0], S.party[1].compute));
  int rc = exchange(-1, false);
  if (rc != LOP_OK) return rc;
  for (int u = 0; u < nl; ++u) {
    for (int d = 0; d < 2; ++d) {
      Party& p = S.party[d];
      const Piece x = xrows(u, d);
      if (x.hi > x.lo) {
        for (hipEvent_t e : p.wait_for[u]) LOP_HIP(hipStreamWaitEvent(p.compute, e, 0));
        LOP_HIP(lop::launch_op(launch[d][u], p.compute, nullptr));
        const double c = cost_seconds(u, d, x.hi - x.lo);
        if (c > 0.0) {
          hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, p.compute, ticks_of(c));
          LOP_HIP(hipGetLastError());
        }
        p.held[u + 1].push_back(x);
      }
      LOP_HIP(hipEventRecord(p.done[u + 1], p.compute));
    }
    rc = exchange(u, false);
    if (rc != LOP_OK) return rc;
  }
  for (hipEvent_t e : S.party[0].wait_for[nl]) LOP_HIP(hipStreamWaitEvent(S.party[0].compute, e, 0));
  LOP_HIP(hipEventRecord(S.t1, S.party[0].compute));
  for (Party& p : S.party) {
    LOP_HIP(hipStreamSynchronize(p.compute));
    LOP_HIP(hipStreamSynchronize(p.link_in));
  }
  if (stats) {
    float ms = 0.f;
    LOP_HIP(hipEventElapsedTime(&ms, S.t0, S.t1));
    stats->total_ms = ms;
    stats->bytes_to_m = bytes_to[0];
    stats->bytes_to_r = bytes_to[1];
    stats->transfers = transfers;
  }
  return LOP_OK;
}
