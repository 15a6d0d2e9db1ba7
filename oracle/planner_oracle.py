"""Oracle of the parallel strategy planner (paper Sec. V): TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.  It shares no code
with the C++ planner of the library.

What it holds is the definition written out: the cost of ONE given strategy exactly as Eq. (3)-(6) state it, and the
optimum of Eq. (2)/(5) under Eq. (6) by enumerating every strategy (small graphs only).  All arithmetic in fp64 on
plain Python numbers.

Model (Sec. V "Simplification"): a chain of k+1 blocks ("nodes"), each a computation sequence with the communication
operator behind it; node v picks one of p partitioning schemes, s_v in [0, p).  Per node and scheme the cost vectors
d^0, d^1 (computation of sub-batch 0 / 1) and c^0, c^1 (communication of sub-batch 0 / 1) exist once for the forward
and once for the backward graph.

Reading taken where the paper leaves the order open: the backward graph visits the nodes in reverse, so "previous
node" in Eq. (3) and the pair of adjacent costs that can no longer overlap in Eq. (4) follow the execution order of
the pass they belong to.  All arrays passed in here are indexed by node in FORWARD order.
"""
from __future__ import annotations

import itertools
from typing import Sequence


def node_cost(d0: Sequence[float], d1: Sequence[float], c0: Sequence[float], c1: Sequence[float]) -> float:
    """Eq. (3): T_V for one pass.  d0[i], d1[i], c0[i], c1[i] are the costs the chosen scheme gives node i, listed in
    the order in which this pass executes the nodes (i = 0 first).

    First term: sub-batch 0 of the first node has nothing to hide behind.  For every later node the computation of
    sub-batch 0 runs beside the previous node's communication of sub-batch 1; for every node the computation of
    sub-batch 1 runs beside the node's own communication of sub-batch 0; each pair costs its maximum.  The last
    communication of sub-batch 1 is exposed.
    """
    k = len(d0) - 1
    total = d0[0]
    for i in range(1, k + 1):
        total += max(d0[i], c1[i - 1])
    for i in range(0, k + 1):
        total += max(d1[i], c0[i])
    total += c1[k]
    return total


def edge_cost(problem: dict, v: int, i: int, j: int) -> float:
    """Eq. (4): cost on the edge between node v (scheme i) and node v+1 (scheme j), forward order.

    i < j: the AllGather is paid in the forward pass, together with what the blocked AllGather no longer lets
    overlap there -- the smaller of node v's communication of sub-batch 1 and node v+1's computation of sub-batch 0.
    i > j: the same in the backward pass, whose execution order is reversed: node v+1 runs first, so the pair is node
    v+1's communication of sub-batch 1 and node v's computation of sub-batch 0.
    """
    if i == j:
        return 0.0
    u = v + 1
    if i < j:
        t_ag = problem["t_ag_f"][v][i][j] if problem.get("t_ag_f") is not None else 0.0
        return t_ag + min(problem["c1_f"][v][i], problem["d0_f"][u][j])
    t_ag = problem["t_ag_b"][v][i][j] if problem.get("t_ag_b") is not None else 0.0
    return t_ag + min(problem["c1_b"][u][j], problem["d0_b"][v][i])


def memory(problem: dict, s: Sequence[int]) -> float:
    """Left side of Eq. (6): temporary buffers of the last node's scheme + model states and saved inputs of all."""
    k = len(s) - 1
    total = problem["m_r"][s[k]]
    for v, sv in enumerate(s):
        total += problem["m_s"][v][sv] + problem["m_t"][v][sv]
    return total


def strategy_cost(problem: dict, s: Sequence[int]) -> dict:
    """Objective of Eq. (5) for strategy s, by its three parts."""
    n = len(s)
    pick = lambda name: [problem[name][v][s[v]] for v in range(n)]
    tv_f = node_cost(pick("d0_f"), pick("d1_f"), pick("c0_f"), pick("c1_f"))
    rev = lambda a: list(reversed(a))
    tv_b = node_cost(rev(pick("d0_b")), rev(pick("d1_b")), rev(pick("c0_b")), rev(pick("c1_b")))
    edges = sum(edge_cost(problem, v, s[v], s[v + 1]) for v in range(n - 1))
    return {"tv_f": tv_f, "tv_b": tv_b, "edges": edges, "total": tv_f + tv_b + edges}


def feasible(problem: dict, s: Sequence[int]) -> bool:
    """Eq. (6) (strict) and, where given, the ties that force adjacent nodes onto one scheme."""
    tie = problem.get("tie")
    if tie is not None and any(tie[v] and s[v] != s[v + 1] for v in range(len(s) - 1)):
        return False
    m = problem.get("m", 0.0)
    return m <= 0 or memory(problem, s) < m


def brute_force(problem: dict):
    """Eq. (2): every strategy in S, the cheapest feasible one.  Returns (strategy, cost) or (None, inf)."""
    n, p = problem["n_nodes"], problem["n_strategies"]
    best, best_cost = None, float("inf")
    for s in itertools.product(range(p), repeat=n):
        if not feasible(problem, s):
            continue
        c = strategy_cost(problem, s)["total"]
        if c < best_cost:
            best, best_cost = list(s), c
    return best, best_cost
