// Local-operation scheduling model (Intra-DP Sec. IV-C) on the host: evaluate a schedule's
// end-to-end time T = s_M(output) (Eq. 2) with the data-dependency recurrence (Eq. 3), and
// search schedules by differential evolution. No GPU work here.
//
// Model (the paper's, with the readings stated where it is silent): a vertex's operations are
// its output rows; a schedule gives each vertex two contiguous intervals x_M, x_R covering all
// rows (they may overlap: replication); the input is whole on M, the result must be whole on
// M; C_D(v) = fixed + per_row * rows (0 if no rows); an edge (u, v) whose consumer rows on D
// read rows of u that D did not produce receives them from the peer after the peer has
// finished u, taking latency + rows * row_bytes(u) / bandwidth. Several parent edges combine
// by max; a device runs its operators one after another in chain order; transfers do not
// queue behind each other (LOP_LINK_INDEPENDENT, Eq. 3 as printed) or share the link as the
// runtime stage does (LOP_LINK_QUEUED, see evaluate_queued). Edges out of a vertex whose output is larger than the raw input
// must carry nothing (transmission-efficiency constraint): counted as violations.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "lop.h"

namespace {

struct Iv {
  int lo, hi;
  int len() const { return hi > lo ? hi - lo : 0; }
};

Iv consumed(const lop_loss_layer_t& L, Iv rows, int parent_rows, bool identity) {
  if (rows.len() == 0) return {0, 0};
  if (identity) return rows;
  const int lo = std::max(rows.lo * L.s - L.p, 0);
  const int hi = std::min((rows.hi - 1) * L.s - L.p + L.d * (L.k - 1) + 1, parent_rows);
  return {lo, std::max(hi, lo)};
}

int missing(Iv need, Iv have) {
  if (need.len() == 0) return 0;
  const int inter = have.len() ? std::max(0, std::min(need.hi, have.hi) - std::max(need.lo, have.lo)) : 0;
  return need.len() - inter;
}

bool covers(const lop_loss_alloc_t& a, int n) {
  const Iv m{a.m_lo, a.m_hi}, r{a.r_lo, a.r_hi};
  for (Iv iv : {m, r})
    if (iv.lo < 0 || iv.lo > iv.hi || iv.hi > n) return false;
  if (m.len() + r.len() == 0) return false;
  // two intervals cover [0, n) iff the one starting first starts at 0, the other starts no
  // later than it ends, and the later end is n
  if (m.len() == 0) return r.lo == 0 && r.hi == n;
  if (r.len() == 0) return m.lo == 0 && m.hi == n;
  const Iv a1 = m.lo <= r.lo ? m : r, a2 = m.lo <= r.lo ? r : m;
  return a1.lo == 0 && a2.lo <= a1.hi && std::max(a1.hi, a2.hi) == n;
}

struct Problem {
  const lop_loss_layer_t* layers;
  int n;
  int in_rows;
  double in_row_bytes, bandwidth, latency;
  int link_model;
};

bool valid_problem(const Problem& P) {
  if (!P.layers || P.n < 1 || P.in_rows < 1 || !(P.bandwidth > 0.0) || P.latency < 0.0) return false;
  if (P.link_model != LOP_LINK_INDEPENDENT && P.link_model != LOP_LINK_QUEUED) return false;
  for (int v = 0; v < P.n; ++v) {
    const lop_loss_layer_t& L = P.layers[v];
    if (L.n_ops < 1 || L.k < 1 || L.s < 1 || L.d < 1 || L.p < 0) return false;
    if (L.input_from < LOP_INPUT || L.input_from >= v) return false;
    if (L.residual_from != LOP_NO_RESIDUAL && (L.residual_from < LOP_INPUT || L.residual_from >= v))
      return false;
    if (L.residual_from != LOP_NO_RESIDUAL) {
      const int pr = L.residual_from == LOP_INPUT ? P.in_rows : P.layers[L.residual_from].n_ops;
      if (pr != L.n_ops) return false;
    }
  }
  return true;
}

// T of a schedule that covers every vertex; s_m (n + 1 values) and s_r (n values) optional.
double evaluate(const Problem& P, const lop_loss_alloc_t* sched, double* s_m, double* s_r,
                int* violations) {
  const int n = P.n;
  std::vector<double> sm(n + 1), sr(n);
  auto rows_of = [&](int u) { return u == LOP_INPUT ? P.in_rows : P.layers[u].n_ops; };
  auto bytes_of = [&](int u) { return u == LOP_INPUT ? P.in_row_bytes : P.layers[u].row_bytes; };
  auto x = [&](int dev, int u) -> Iv {
    if (u == LOP_INPUT) return dev == 0 ? Iv{0, P.in_rows} : Iv{0, 0};
    return dev == 0 ? Iv{sched[u].m_lo, sched[u].m_hi} : Iv{sched[u].r_lo, sched[u].r_hi};
  };
  auto cost = [&](int dev, int u) -> double {
    if (u == LOP_INPUT) return 0.0;
    const int rows = x(dev, u).len();
    if (rows == 0) return 0.0;
    const lop_loss_layer_t& L = P.layers[u];
    return dev == 0 ? L.cm_fixed + L.cm_row * rows : L.cr_fixed + L.cr_row * rows;
  };
  auto start = [&](int dev, int u) -> double {
    if (u == LOP_INPUT) return 0.0;
    return dev == 0 ? sm[u] : sr[u];
  };
  const double raw_input = (double)P.in_rows * P.in_row_bytes;
  int viol = 0;
  struct Edge { int u; Iv need; };
  auto ready = [&](int dev, const Edge* edges, int n_edges, int prev) -> double {
    const int peer = 1 - dev;
    double t = 0.0;
    if (prev >= 0) t = start(dev, prev) + cost(dev, prev);
    for (int e = 0; e < n_edges; ++e) {
      const int u = edges[e].u;
      double local = start(dev, u) + cost(dev, u);
      const int miss = missing(edges[e].need, x(dev, u));
      if (miss) {
        const double arrive = start(peer, u) + cost(peer, u) + P.latency + miss * bytes_of(u) / P.bandwidth;
        local = std::max(local, arrive);
        if ((double)rows_of(u) * bytes_of(u) > raw_input) ++viol;
      }
      t = std::max(t, local);
    }
    return t;
  };
  for (int v = 0; v < n; ++v) {
    const lop_loss_layer_t& L = P.layers[v];
    for (int dev = 0; dev < 2; ++dev) {
      const Iv mine = x(dev, v);
      Edge edges[2];
      int ne = 0;
      edges[ne++] = {L.input_from, consumed(L, mine, rows_of(L.input_from), false)};
      if (L.residual_from != LOP_NO_RESIDUAL)
        edges[ne++] = {L.residual_from, consumed(L, mine, rows_of(L.residual_from), true)};
      (dev == 0 ? sm[v] : sr[v]) = ready(dev, edges, ne, v - 1);
    }
  }
  const Edge out{n - 1, Iv{0, P.layers[n - 1].n_ops}};
  sm[n] = ready(0, &out, 1, n - 1);
  if (s_m) std::copy(sm.begin(), sm.end(), s_m);
  if (s_r) std::copy(sr.begin(), sr.end(), s_r);
  if (violations) *violations = viol;
  return sm[n];
}

// need minus the union of held (sorted disjoint pieces; at most a handful)
void minus(Iv need, const std::vector<Iv>& held, std::vector<Iv>& out) {
  out.clear();
  if (need.len()) out.push_back(need);
  std::vector<Iv> nxt;
  for (const Iv& h : held) {
    if (!h.len()) continue;
    nxt.clear();
    for (const Iv& p : out) {
      if (h.hi <= p.lo || h.lo >= p.hi) { nxt.push_back(p); continue; }
      if (p.lo < h.lo) nxt.push_back({p.lo, h.lo});
      if (h.hi < p.hi) nxt.push_back({h.hi, p.hi});
    }
    out.swap(nxt);
  }
}

// The same model with the link shared the way the runtime stage shares it (Sec. IV-D, Alg. 1
// and 2): after every vertex u the rows its consumers on the other device will read travel as
// messages, edge by edge; a message occupies its direction of the link for latency + bytes /
// bandwidth, so messages of one direction queue in issue order; rows a device already holds
// are not sent again; a consumer waits only for its own messages.
double evaluate_queued(const Problem& P, const lop_loss_alloc_t* sched, double* s_m, double* s_r,
                       int* violations) {
  const int n = P.n;
  auto rows_of = [&](int u) { return u == LOP_INPUT ? P.in_rows : P.layers[u].n_ops; };
  auto bytes_of = [&](int u) { return u == LOP_INPUT ? P.in_row_bytes : P.layers[u].row_bytes; };
  auto x = [&](int dev, int v) -> Iv {
    return dev == 0 ? Iv{sched[v].m_lo, sched[v].m_hi} : Iv{sched[v].r_lo, sched[v].r_hi};
  };
  const double raw_input = (double)P.in_rows * P.in_row_bytes;
  std::vector<std::vector<Iv>> held[2];
  std::vector<double> finish[2], start[2], arrive[2];
  for (int d = 0; d < 2; ++d) {
    held[d].assign(n + 1, {});
    finish[d].assign(n + 1, 0.0);  // [u + 1]
    start[d].assign(n, 0.0);
    arrive[d].assign(n + 1, 0.0);  // [consumer]; n = the result
  }
  held[0][0].push_back({0, P.in_rows});
  double link_free[2] = {0.0, 0.0};  // direction into that device
  int viol = 0;
  std::vector<Iv> pieces;
  auto exchange = [&](int u) {
    for (int v = 0; v <= n; ++v) {
      bool kinds[2];
      int nk = 0;
      if (v == n) {
        if (u == n - 1) kinds[nk++] = true;
      } else {
        if (P.layers[v].input_from == u) kinds[nk++] = false;
        if (P.layers[v].residual_from == u) kinds[nk++] = true;
      }
      for (int k = 0; k < nk; ++k)
        for (int d = 0; d < 2; ++d) {
          Iv need;
          if (v == n) need = d == 0 ? Iv{0, rows_of(u)} : Iv{0, 0};
          else need = consumed(P.layers[v], x(d, v), rows_of(u), kinds[k]);
          minus(need, held[d][u + 1], pieces);
          for (const Iv& pc : pieces) {
            const double begin = std::max(finish[1 - d][u + 1], link_free[d]);
            const double done = begin + P.latency + pc.len() * bytes_of(u) / P.bandwidth;
            link_free[d] = done;
            arrive[d][v] = std::max(arrive[d][v], done);
            held[d][u + 1].push_back(pc);
            if ((double)rows_of(u) * bytes_of(u) > raw_input) ++viol;
          }
        }
    }
  };
  exchange(LOP_INPUT);
  for (int u = 0; u < n; ++u) {
    const lop_loss_layer_t& L = P.layers[u];
    for (int d = 0; d < 2; ++d) {
      double s = arrive[d][u];
      if (u > 0) s = std::max(s, finish[d][u]);
      start[d][u] = s;
      const int rows = x(d, u).len();
      double c = 0.0;
      if (rows) {
        c = d == 0 ? L.cm_fixed + L.cm_row * rows : L.cr_fixed + L.cr_row * rows;
        held[d][u + 1].push_back(x(d, u));
      }
      finish[d][u + 1] = s + c;
    }
    exchange(u);
  }
  const double t_out = std::max(finish[0][n], arrive[0][n]);
  if (s_m) {
    std::copy(start[0].begin(), start[0].end(), s_m);
    s_m[n] = t_out;
  }
  if (s_r) std::copy(start[1].begin(), start[1].end(), s_r);
  if (violations) *violations = viol;
  return t_out;
}

double evaluate_any(const Problem& P, const lop_loss_alloc_t* sched, double* s_m, double* s_r,
                    int* violations) {
  return P.link_model == LOP_LINK_QUEUED ? evaluate_queued(P, sched, s_m, s_r, violations)
                                         : evaluate(P, sched, s_m, s_r, violations);
}

// splitmix64: the differential evolution's only source of randomness
struct Rng {
  uint64_t s;
  uint64_t next() {
    uint64_t z = (s += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
  }
  double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
  int below(int n) { return (int)(next() % (uint64_t)n); }
};

// Decision vector: per vertex a in [0, 1] (share of leading rows on M) and r in [0, 1] (how
// far R's interval reaches back into M's rows): x_M = [0, A), x_R = [B, n), B <= A, so every
// vector decodes to a schedule that satisfies the partitioning and contiguity constraints.
void decode(const Problem& P, const std::vector<double>& g, lop_loss_alloc_t* out) {
  for (int v = 0; v < P.n; ++v) {
    const int n = P.layers[v].n_ops;
    const int A = std::min(n, std::max(0, (int)std::lround(g[2 * v] * n)));
    const int B = std::min(A, std::max(0, (int)std::lround((1.0 - g[2 * v + 1]) * A)));
    out[v].m_lo = 0; out[v].m_hi = A;
    out[v].r_lo = B; out[v].r_hi = n;
    if (A == n && B == n) out[v].r_lo = out[v].r_hi = 0;
  }
}

double fitness(const Problem& P, const std::vector<double>& g, std::vector<lop_loss_alloc_t>& tmp) {
  decode(P, g, tmp.data());
  int viol = 0;
  const double t = evaluate_any(P, tmp.data(), nullptr, nullptr, &viol);
  // a schedule that breaks the transmission-efficiency constraint loses against every one
  // that keeps it, and among such schedules fewer violations win
  return viol ? 1e30 * viol + t : t;
}

}  // namespace

extern "C" {

int lop_loss_eval(const lop_loss_layer_t* layers, int n_layers, int in_rows, double in_row_bytes,
                  double bandwidth, double latency, const lop_loss_alloc_t* sched, double* T,
                  double* s_m, double* s_r, int* violations, int link_model) {
  const Problem P{layers, n_layers, in_rows, in_row_bytes, bandwidth, latency, link_model};
  if (!sched || !T || !valid_problem(P)) return LOP_ERR_INVALID_ARG;
  for (int v = 0; v < n_layers; ++v)
    if (!covers(sched[v], layers[v].n_ops)) return LOP_ERR_BAND_RANGE;
  *T = evaluate_any(P, sched, s_m, s_r, violations);
  return LOP_OK;
}

int lop_loss_solve(const lop_loss_layer_t* layers, int n_layers, int in_rows, double in_row_bytes,
                   double bandwidth, double latency, int population, int generations,
                   unsigned long long seed, lop_loss_alloc_t* best, double* T, int* violations,
                   int link_model) {
  const Problem P{layers, n_layers, in_rows, in_row_bytes, bandwidth, latency, link_model};
  if (!best || !T || !valid_problem(P) || generations < 0) return LOP_ERR_INVALID_ARG;
  const int dim = 2 * n_layers;
  const int np = std::max(population > 0 ? population : 10 * dim, 8);
  const double F = 0.6, CR = 0.9;  // DE/rand/1/bin
  Rng rng{seed};
  std::vector<lop_loss_alloc_t> tmp((size_t)n_layers);
  std::vector<std::vector<double>> pop((size_t)np, std::vector<double>((size_t)dim));
  std::vector<double> fit((size_t)np);
  for (int i = 0; i < np; ++i) {
    for (double& g : pop[i]) g = rng.uniform();
    // seed the population with the two one-device schedules and an even split
    if (i < 3)
      for (int v = 0; v < n_layers; ++v) {
        pop[i][2 * v] = i == 0 ? 1.0 : (i == 1 ? 0.0 : 0.5);
        pop[i][2 * v + 1] = 0.0;
      }
    fit[i] = fitness(P, pop[i], tmp);
  }
  std::vector<double> trial((size_t)dim);
  for (int gen = 0; gen < generations; ++gen)
    for (int i = 0; i < np; ++i) {
      int a, b, c;
      do a = rng.below(np); while (a == i);
      do b = rng.below(np); while (b == i || b == a);
      do c = rng.below(np); while (c == i || c == a || c == b);
      const int forced = rng.below(dim);
      for (int j = 0; j < dim; ++j) {
        double g = pop[i][j];
        if (j == forced || rng.uniform() < CR) g = pop[a][j] + F * (pop[b][j] - pop[c][j]);
        trial[j] = std::min(1.0, std::max(0.0, g));
      }
      const double f = fitness(P, trial, tmp);
      if (f <= fit[i]) {
        pop[i] = trial;
        fit[i] = f;
      }
    }
  const int bi = (int)(std::min_element(fit.begin(), fit.end()) - fit.begin());
  decode(P, pop[bi], best);
  *T = evaluate_any(P, best, nullptr, nullptr, violations);
  return LOP_OK;
}

}  // extern "C"
