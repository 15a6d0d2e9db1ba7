"""Pins of the planner oracle (paper Sec. V, Eq. (3)-(6)) against things other than itself: a two-stream timeline
simulation written here from the schedule's dependencies (Sec. IV-C / Sec. V-B), closed forms, and a case worked by
hand.  No GPU."""
import random

import pytest

from oracle import planner_oracle as po


def timeline_makespan(d0, d1, c0, c1):
    """Discrete-event run of one pass: the computation stream executes d_0^0, d_0^1, d_1^0, d_1^1, ... in order, the
    communication stream c_0^0, c_0^1, c_1^0, ... in order; a communication starts when its computation is done, and
    node i+1's computation of a sub-batch needs node i's communication of that sub-batch (Sec. IV-C: while one
    sub-batch computes, the other communicates)."""
    k = len(d0) - 1
    comp_free = comm_free = 0.0
    comm_done = {(-1, 0): 0.0, (-1, 1): 0.0}
    for i in range(k + 1):
        for x, d, c in ((0, d0[i], c0[i]), (1, d1[i], c1[i])):
            start = max(comp_free, comm_done[(i - 1, x)])
            comp_free = start + d
            cstart = max(comm_free, comp_free)
            comm_free = cstart + c
            comm_done[(i, x)] = comm_free
    return max(comp_free, comm_free)


def rand_pass(rng, k, dscale, cscale):
    f = lambda s: [rng.uniform(0.1, 1.0) * s for _ in range(k + 1)]
    return f(dscale), f(dscale), f(cscale), f(cscale)


def test_node_cost_closed_forms():
    rng = random.Random(1)
    d0, d1, c0, c1 = rand_pass(rng, 5, 1.0, 1.0)
    z = [0.0] * 6
    assert po.node_cost(d0, d1, z, z) == pytest.approx(sum(d0) + sum(d1), rel=1e-15)      # nothing to wait for
    assert po.node_cost(z, z, c0, c1) == pytest.approx(sum(c0) + sum(c1), rel=1e-15)      # nothing to hide behind
    # single node: d^0, then max(d^1, c^0), then the exposed c^1
    assert po.node_cost([2.0], [3.0], [5.0], [7.0]) == 2.0 + 5.0 + 7.0
    assert po.node_cost([2.0], [3.0], [1.0], [7.0]) == 2.0 + 3.0 + 7.0


def test_node_cost_worked_by_hand():
    # three nodes; by Eq. (3):
    #   d0_0                         = 4
    #   max(d0_1, c1_0) = max(3, 5)  = 5      max(d0_2, c1_1) = max(6, 2) = 6
    #   max(d1_0, c0_0) = max(4, 1)  = 4      max(d1_1, c0_1) = max(3, 7) = 7      max(d1_2, c0_2) = max(6, 6) = 6
    #   c1_2                         = 9
    assert po.node_cost([4, 3, 6], [4, 3, 6], [1, 7, 6], [5, 2, 9]) == 4 + 5 + 6 + 4 + 7 + 6 + 9


@pytest.mark.parametrize("seed", range(8))
def test_node_cost_against_timeline(seed):
    rng = random.Random(seed)
    k = rng.randint(1, 7)
    # communication always hidden: the estimate is exact, sum of all computation + the last communication
    d0, d1, c0, c1 = rand_pass(rng, k, 1.0, 0.09)
    assert po.node_cost(d0, d1, c0, c1) == pytest.approx(timeline_makespan(d0, d1, c0, c1), rel=1e-12)
    assert po.node_cost(d0, d1, c0, c1) == pytest.approx(sum(d0) + sum(d1) + c1[-1], rel=1e-12)
    # communication always dominant: exact again, first computation + all communication
    d0, d1, c0, c1 = rand_pass(rng, k, 0.09, 1.0)
    assert po.node_cost(d0, d1, c0, c1) == pytest.approx(timeline_makespan(d0, d1, c0, c1), rel=1e-12)
    # mixed: pairing by max never underestimates the timeline, and never exceeds running everything back to back
    d0, d1, c0, c1 = rand_pass(rng, k, 1.0, 1.0)
    est = po.node_cost(d0, d1, c0, c1)
    assert timeline_makespan(d0, d1, c0, c1) <= est * (1 + 1e-12)
    assert est <= sum(d0) + sum(d1) + sum(c0) + sum(c1)


def two_node_problem():
    # p = 2 schemes; all vectors [node][scheme]
    return {
        "n_nodes": 2, "n_strategies": 2,
        "d0_f": [[10, 6], [12, 7]], "d1_f": [[10, 6], [12, 7]], "c0_f": [[1, 3], [1, 4]], "c1_f": [[2, 5], [1, 4]],
        "d0_b": [[20, 11], [24, 13]], "d1_b": [[20, 11], [24, 13]], "c0_b": [[1, 3], [1, 4]], "c1_b": [[2, 5], [3, 8]],
        "t_ag_f": [[[0, 0.5], [0.25, 0]]], "t_ag_b": [[[0, 0.75], [1.5, 0]]],
        "m_s": [[8, 4], [8, 4]], "m_t": [[1, 1], [1, 1]], "m_r": [3, 2], "m": 0.0,
    }


def test_edge_cost_by_hand():
    p = two_node_problem()
    assert po.edge_cost(p, 0, 0, 0) == 0.0 and po.edge_cost(p, 0, 1, 1) == 0.0
    # scheme 0 -> 1 (i < j): forward AllGather 0.5 + min(c1_f[node 0][0], d0_f[node 1][1]) = 0.5 + min(2, 7)
    assert po.edge_cost(p, 0, 0, 1) == 0.5 + 2
    # scheme 1 -> 0 (i > j): backward AllGather 1.5 + min(c1_b[node 1][0], d0_b[node 0][1]) = 1.5 + min(3, 11)
    assert po.edge_cost(p, 0, 1, 0) == 1.5 + 3


def test_strategy_cost_and_memory_by_hand():
    p = two_node_problem()
    c = po.strategy_cost(p, [1, 0])
    # forward, order node 0 then 1:  d0 = [6, 12], d1 = [6, 12], c0 = [3, 1], c1 = [5, 1]
    #   6 + max(12, 5) + max(6, 3) + max(12, 1) + 1 = 37
    assert c["tv_f"] == 37
    # backward, order node 1 then 0: d0 = [24, 11], d1 = [24, 11], c0 = [1, 3], c1 = [3, 5]
    #   24 + max(11, 3) + max(24, 1) + max(11, 3) + 5 = 75
    assert c["tv_b"] == 75
    assert c["edges"] == 4.5 and c["total"] == 37 + 75 + 4.5
    # Eq. (6): m_r of the last node's scheme + per-node states and saved inputs
    assert po.memory(p, [1, 0]) == 3 + (4 + 1) + (8 + 1)
    assert po.memory(p, [0, 1]) == 2 + (8 + 1) + (4 + 1)


def test_brute_force_memory_and_ties():
    p = two_node_problem()
    s, c = po.brute_force(p)
    assert c == min(po.strategy_cost(p, [a, b])["total"] for a in (0, 1) for b in (0, 1))
    assert s == [1, 1]                      # the cheaper scheme everywhere, no reshard
    p["m"] = 12.0                           # [1,1] needs 2 + 5 + 5 = 12: the bound is strict, so nothing fits
    assert po.brute_force(p) == (None, float("inf"))
    p["m"] = 12.5
    assert po.brute_force(p)[0] == [1, 1]
    # costs that favour scheme 0, memory that only admits one node on it
    q = two_node_problem()
    for name in ("d0_f", "d1_f", "d0_b", "d1_b"):
        q[name] = [[1, 9], [1, 9]]
    q["m"] = 17.5                           # [0,0] needs 3+9+9 = 21; [0,1]: 2+9+5 = 16; [1,0]: 3+5+9 = 17
    s, _ = po.brute_force(q)
    assert s in ([0, 1], [1, 0]) and po.memory(q, s) < 17.5
    q["tie"] = [1]                          # adjacent nodes forced onto one scheme: only [1,1] fits
    assert po.brute_force(q)[0] == [1, 1]
