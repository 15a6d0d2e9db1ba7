"""ctypes binding of the parallel strategy planner (include/oases_planner.h): argument marshalling only.

A problem is a dict with the keys of `oases_plan_problem`; array values are nested lists or numpy arrays indexed
[node][scheme] (AllGather: [edge][i][j]; m_r: [scheme]; tie: [edge]), all in forward node order.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import binding as B

_D = C.POINTER(C.c_double)
_COST = ("d0_f", "d1_f", "c0_f", "c1_f", "d0_b", "d1_b", "c0_b", "c1_b")
EINFEASIBLE = -6


class PlanProblem(C.Structure):
    _fields_ = ([("n_nodes", C.c_int32), ("n_strategies", C.c_int32)] + [(n, _D) for n in _COST] +
                [("t_ag_f", _D), ("t_ag_b", _D), ("m_s", _D), ("m_t", _D), ("m_r", _D), ("m", C.c_double),
                 ("tie", C.POINTER(C.c_uint8))])


B.lib.oases_plan_cost.restype = C.c_int
B.lib.oases_plan_cost.argtypes = [C.POINTER(PlanProblem), C.POINTER(C.c_int32), _D, _D]
B.lib.oases_plan_solve.restype = C.c_int
B.lib.oases_plan_solve.argtypes = [C.POINTER(PlanProblem), C.POINTER(C.c_int32), _D, _D]


def _marshal(problem: dict):
    """dict -> (PlanProblem, list of arrays that must stay alive)."""
    n, p = int(problem["n_nodes"]), int(problem["n_strategies"])
    q, keep = PlanProblem(), []
    q.n_nodes, q.n_strategies, q.m = n, p, float(problem.get("m", 0.0) or 0.0)

    def put(name, shape, dtype=np.float64, ctype=_D):
        v = problem.get(name)
        if v is None:
            return
        a = np.ascontiguousarray(np.asarray(v, dtype=dtype))
        if a.size == 0 and 0 in shape:
            return
        if a.shape != shape:
            raise ValueError(f"{name}: shape {a.shape}, expected {shape}")
        keep.append(a)
        setattr(q, name, a.ctypes.data_as(ctype))

    for name in _COST + ("m_s", "m_t"):
        put(name, (n, p))
    put("m_r", (p,))
    put("t_ag_f", (n - 1, p, p))
    put("t_ag_b", (n - 1, p, p))
    put("tie", (n - 1,), np.uint8, C.POINTER(C.c_uint8))
    return q, keep


def plan_cost(problem: dict, strategy) -> dict:
    q, keep = _marshal(problem)
    s = (C.c_int32 * q.n_nodes)(*[int(x) for x in strategy])
    parts, mem = (C.c_double * 4)(), C.c_double()
    B.check(B.lib.oases_plan_cost(C.byref(q), s, parts, C.byref(mem)))
    return {"tv_f": parts[0], "tv_b": parts[1], "edges": parts[2], "total": parts[3], "memory": mem.value}


def plan_solve(problem: dict):
    """Returns (strategy list, cost, memory), or (None, inf, None) if no strategy is feasible."""
    q, keep = _marshal(problem)
    s = (C.c_int32 * q.n_nodes)()
    cost, mem = C.c_double(), C.c_double()
    rc = B.lib.oases_plan_solve(C.byref(q), s, C.byref(cost), C.byref(mem))
    if rc == EINFEASIBLE:
        return None, float("inf"), None
    B.check(rc)
    return list(s), cost.value, mem.value
