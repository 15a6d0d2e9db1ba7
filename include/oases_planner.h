/*
 * oases_planner.h -- C ABI of the parallel strategy planner (paper Sec. V).  HOST ONLY: every pointer is host
 * memory owned by the caller, no GPU is touched, nothing is allocated that outlives a call.
 *
 * The model graph is a chain of k+1 blocks ("nodes", Sec. V "Simplification": a computation sequence and the
 * communication operator behind it), listed in FORWARD order.  Node v picks one of p partitioning schemes,
 * s_v in [0, p) (the paper's one-hot vectors s_v, Eq. (2)); schemes are ordered as Eq. (4) orders them: an edge
 * whose scheme index rises pays its AllGather in the forward pass, one whose index falls pays it in the backward
 * pass.  Costs are doubles in any one unit of time, memory in any one unit of size.
 *
 * Objective, Eq. (5): T_V(d(F), c(F)) + T_V(d(B), c(B)) + sum over edges of R, with T_V of Eq. (3) and R of
 * Eq. (4), under the memory bound of Eq. (6).  Reading where the paper leaves the order open: the backward pass
 * visits the nodes in reverse, so "previous node" in Eq. (3) and the adjacent pair of Eq. (4) follow the
 * execution order of the pass they belong to.  The graph is a chain, so the optimum is found exactly by dynamic
 * programming over (node, scheme) with the non-dominated (cost, memory) pairs kept per state; no ILP solver.
 *
 * Errors: OASES_ENULL (a required pointer is NULL), OASES_EINVAL (sizes, negative or non-finite entries),
 * OASES_EINFEASIBLE (no strategy satisfies Eq. (6) and the ties); text in oases_last_error().
 */
#ifndef OASES_PLANNER_H
#define OASES_PLANNER_H

#include <stdint.h>

#include "oases.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t n_nodes;      /* k+1 >= 1 */
  int32_t n_strategies; /* p >= 1 */
  /* cost vectors of Eq. (3), each [n_nodes][p] row-major: computation of sub-batch 0 / 1 and communication of
   * sub-batch 0 / 1 of a node under a scheme, for the forward (_f) and the backward (_b) graph */
  const double *d0_f, *d1_f, *c0_f, *c1_f;
  const double *d0_b, *d1_b, *c0_b, *c1_b;
  /* T_AG of Eq. (4): [n_nodes-1][p][p], entry [v][i][j] = AllGather time between node v on scheme i and node v+1
   * on scheme j, paid in the forward pass (i < j, t_ag_f) or the backward pass (i > j, t_ag_b); other entries
   * are ignored.  NULL = all zero. */
  const double *t_ag_f, *t_ag_b;
  /* Eq. (6): model states and saved inputs per node and scheme [n_nodes][p], temporary buffers per scheme [p]
   * (counted once, for the last node's scheme), capacity m.  m <= 0: no memory bound (the three arrays may then
   * be NULL). */
  const double *m_s, *m_t, *m_r;
  double m;
  /* optional [n_nodes-1]: tie[v] != 0 forces nodes v and v+1 onto one scheme (e.g. the blocks of one layer).
   * NULL = no ties. */
  const uint8_t *tie;
} oases_plan_problem;

/* Cost of one strategy as Eq. (3)-(5) define it.  strategy: [n_nodes] scheme indices.  parts (optional):
 * [4] = { T_V forward, T_V backward, sum of edge costs, total }.  memory (optional): left side of Eq. (6), 0 if
 * the problem has no memory arrays.  Does not check feasibility. */
int oases_plan_cost(const oases_plan_problem *p, const int32_t *strategy, double *parts, double *memory);

/* The cheapest feasible strategy (Eq. (2)).  strategy: [n_nodes] out.  cost / memory (optional): its objective
 * value and the left side of Eq. (6).  Among strategies of equal cost the one with less memory wins. */
int oases_plan_solve(const oases_plan_problem *p, int32_t *strategy, double *cost, double *memory);

#ifdef __cplusplus
}
#endif
#endif
