// Parallel strategy planner (paper Sec. V): exact optimum of Eq. (5) under Eq. (6) on a chain of blocks.
//
// Eq. (3) couples a node only with its neighbour (the computation of sub-batch 0 runs beside the neighbour's
// communication of sub-batch 1) and Eq. (4) is an edge cost, so the objective is a sum of per-node and
// per-adjacent-pair terms: a shortest path over (node, scheme) layers.  The memory bound of Eq. (6) adds a second
// additive quantity; per (node, scheme) the labels (cost, memory) that no other label beats in both are kept, which
// keeps the search exact.  Host code only.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "../../include/oases_planner.h"

namespace oases {
void set_error(const char* fmt, ...);
}
using oases::set_error;

namespace {

struct View {
  const oases_plan_problem& q;
  int n, p;
  double at(const double* a, int v, int j) const { return a[(size_t)v * p + j]; }
  double ag(const double* a, int v, int i, int j) const { return a ? a[((size_t)v * p + i) * p + j] : 0.0; }
  bool bounded() const { return q.m > 0; }

  // terms of Eq. (3) that involve node v alone: sub-batch 1 computes beside the node's own communication of
  // sub-batch 0 (both passes); the pass that starts at v pays its d^0 in full, the pass that ends at v its c^1
  double unary(int v, int j) const {
    double t = std::max(at(q.d1_f, v, j), at(q.c0_f, v, j)) + std::max(at(q.d1_b, v, j), at(q.c0_b, v, j));
    if (v == 0) t += at(q.d0_f, v, j) + at(q.c1_b, v, j);
    if (v == n - 1) t += at(q.c1_f, v, j) + at(q.d0_b, v, j);
    return t;
  }
  // Eq. (4) between node v on scheme i and node v+1 on scheme j
  double edge(int v, int i, int j) const {
    if (i == j) return 0.0;
    if (i < j) return ag(q.t_ag_f, v, i, j) + std::min(at(q.c1_f, v, i), at(q.d0_f, v + 1, j));
    return ag(q.t_ag_b, v, i, j) + std::min(at(q.c1_b, v + 1, j), at(q.d0_b, v, i));
  }
  // terms that involve nodes v and v+1: forward, v+1 computes sub-batch 0 beside v's communication of sub-batch 1;
  // backward the roles are swapped; plus the edge
  double pair(int v, int i, int j) const {
    return std::max(at(q.d0_f, v + 1, j), at(q.c1_f, v, i)) + std::max(at(q.d0_b, v, i), at(q.c1_b, v + 1, j)) + edge(v, i, j);
  }
  double mem(int v, int j) const {
    if (!q.m_s) return 0.0;
    return at(q.m_s, v, j) + at(q.m_t, v, j) + (v == n - 1 ? q.m_r[j] : 0.0);
  }
};

int validate(const oases_plan_problem* q) {
  if (!q) { set_error("planner: NULL problem"); return OASES_ENULL; }
  if (q->n_nodes < 1 || q->n_strategies < 1 || q->n_nodes > (1 << 20) || q->n_strategies > 64) {
    set_error("planner: n_nodes=%d, n_strategies=%d out of range", q->n_nodes, q->n_strategies);
    return OASES_EINVAL;
  }
  const double* need[] = {q->d0_f, q->d1_f, q->c0_f, q->c1_f, q->d0_b, q->d1_b, q->c0_b, q->c1_b};
  for (const double* a : need)
    if (!a) { set_error("planner: NULL cost vector"); return OASES_ENULL; }
  const bool any_mem = q->m_s || q->m_t || q->m_r;
  if ((q->m > 0 || any_mem) && !(q->m_s && q->m_t && q->m_r)) { set_error("planner: memory bound needs m_s, m_t and m_r"); return OASES_ENULL; }
  const size_t np = (size_t)q->n_nodes * q->n_strategies;
  auto ok = [](const double* a, size_t cnt) {
    for (size_t i = 0; i < cnt; i++)
      if (!(a[i] >= 0.0) || !std::isfinite(a[i])) return false;
    return true;
  };
  for (const double* a : need)
    if (!ok(a, np)) { set_error("planner: cost entries must be finite and >= 0"); return OASES_EINVAL; }
  if (q->m_s && (!ok(q->m_s, np) || !ok(q->m_t, np) || !ok(q->m_r, (size_t)q->n_strategies))) {
    set_error("planner: memory entries must be finite and >= 0");
    return OASES_EINVAL;
  }
  const size_t ne = (size_t)(q->n_nodes - 1) * q->n_strategies * q->n_strategies;
  if ((q->t_ag_f && !ok(q->t_ag_f, ne)) || (q->t_ag_b && !ok(q->t_ag_b, ne))) { set_error("planner: AllGather entries must be finite and >= 0"); return OASES_EINVAL; }
  if (!std::isfinite(q->m)) { set_error("planner: capacity not finite"); return OASES_EINVAL; }
  return 0;
}

struct Label {
  double cost, mem;
  int32_t prev_scheme, prev_label;
};

// keep the labels no other label beats: ascending cost, strictly descending memory
void prune(std::vector<Label>& f, bool bounded) {
  std::sort(f.begin(), f.end(), [](const Label& a, const Label& b) {
    if (a.cost != b.cost) return a.cost < b.cost;
    if (a.mem != b.mem) return a.mem < b.mem;
    return a.prev_scheme < b.prev_scheme;
  });
  if (f.empty()) return;
  if (!bounded) { f.resize(1); return; }
  size_t w = 1;
  double best_mem = f[0].mem;
  for (size_t r = 1; r < f.size(); r++)
    if (f[r].mem < best_mem) { best_mem = f[r].mem; f[w++] = f[r]; }
  f.resize(w);
}

}  // namespace

extern "C" int oases_plan_cost(const oases_plan_problem* q, const int32_t* s, double* parts, double* memory) {
  if (int rc = validate(q)) return rc;
  if (!s) { set_error("planner: NULL strategy"); return OASES_ENULL; }
  const View V{*q, q->n_nodes, q->n_strategies};
  const int n = V.n;
  for (int v = 0; v < n; v++)
    if (s[v] < 0 || s[v] >= V.p) { set_error("planner: strategy[%d]=%d outside [0,%d)", v, s[v], V.p); return OASES_EINVAL; }
  // Eq. (3), forward order 0..k
  double tf = V.at(q->d0_f, 0, s[0]);
  for (int v = 1; v < n; v++) tf += std::max(V.at(q->d0_f, v, s[v]), V.at(q->c1_f, v - 1, s[v - 1]));
  for (int v = 0; v < n; v++) tf += std::max(V.at(q->d1_f, v, s[v]), V.at(q->c0_f, v, s[v]));
  tf += V.at(q->c1_f, n - 1, s[n - 1]);
  // Eq. (3), backward order k..0
  double tb = V.at(q->d0_b, n - 1, s[n - 1]);
  for (int v = n - 2; v >= 0; v--) tb += std::max(V.at(q->d0_b, v, s[v]), V.at(q->c1_b, v + 1, s[v + 1]));
  for (int v = n - 1; v >= 0; v--) tb += std::max(V.at(q->d1_b, v, s[v]), V.at(q->c0_b, v, s[v]));
  tb += V.at(q->c1_b, 0, s[0]);
  double te = 0.0;
  for (int v = 0; v + 1 < n; v++) te += V.edge(v, s[v], s[v + 1]);
  if (parts) { parts[0] = tf; parts[1] = tb; parts[2] = te; parts[3] = tf + tb + te; }
  if (memory) {
    double m = 0.0;
    for (int v = 0; v < n; v++) m += V.mem(v, s[v]);
    *memory = m;
  }
  return 0;
}

extern "C" int oases_plan_solve(const oases_plan_problem* q, int32_t* strategy, double* cost, double* memory) {
  if (int rc = validate(q)) return rc;
  if (!strategy) { set_error("planner: NULL strategy"); return OASES_ENULL; }
  const View V{*q, q->n_nodes, q->n_strategies};
  const int n = V.n, p = V.p;
  const bool bounded = V.bounded();
  constexpr size_t kMaxLabels = 1u << 22;

  std::vector<std::vector<std::vector<Label>>> front(n, std::vector<std::vector<Label>>(p));
  for (int j = 0; j < p; j++) {
    Label l{V.unary(0, j), V.mem(0, j), -1, -1};
    if (!bounded || l.mem < q->m) front[0][j].push_back(l);
  }
  size_t total_labels = 0;
  for (int v = 1; v < n; v++) {
    for (int j = 0; j < p; j++) {
      std::vector<Label>& out = front[v][j];
      const double u = V.unary(v, j), mj = V.mem(v, j);
      for (int i = 0; i < p; i++) {
        if (q->tie && q->tie[v - 1] && i != j) continue;
        const std::vector<Label>& in = front[v - 1][i];
        if (in.empty()) continue;
        const double pc = V.pair(v - 1, i, j);
        for (size_t a = 0; a < in.size(); a++) {
          Label l{in[a].cost + pc + u, in[a].mem + mj, i, (int32_t)a};
          if (bounded && !(l.mem < q->m)) continue;  // memory only grows along the chain
          out.push_back(l);
        }
      }
      prune(out, bounded);
      total_labels += out.size();
      if (total_labels > kMaxLabels) { set_error("planner: more than %zu non-dominated (cost, memory) labels", kMaxLabels); return OASES_EINVAL; }
    }
  }
  int bj = -1, bl = -1;
  for (int j = 0; j < p; j++)
    for (size_t a = 0; a < front[n - 1][j].size(); a++) {
      const Label& l = front[n - 1][j][a];
      if (bj < 0) { bj = j; bl = (int)a; continue; }
      const Label& b = front[n - 1][bj][bl];
      if (l.cost < b.cost || (l.cost == b.cost && l.mem < b.mem)) { bj = j; bl = (int)a; }
    }
  if (bj < 0) { set_error("planner: no strategy satisfies the memory bound %g and the ties", q->m); return OASES_EINFEASIBLE; }
  if (cost) *cost = front[n - 1][bj][bl].cost;
  if (memory) *memory = front[n - 1][bj][bl].mem;
  for (int v = n - 1; v >= 0; v--) {
    strategy[v] = bj;
    const Label& l = front[v][bj][bl];
    bj = l.prev_scheme;
    bl = l.prev_label;
  }
  return 0;
}
