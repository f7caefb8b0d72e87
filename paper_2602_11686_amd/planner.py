"""ctypes binding of the host-side planner in libmoe.so: same names as include/moe_planner.h.

Argument marshalling only (numpy host arrays in, numpy host arrays out); every algorithm runs in
the C++ library.  There is no Python fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

from .binding import MoeError, lib

PLANNER_EXPORTS = ["moe_plan_replica_allocation", "moe_plan_expert_relocation", "moe_plan_lite_routing",
                   "moe_plan_time_cost", "moe_plan_expert_layout", "moe_plan_dispatch_table"]


class _CPlanShape(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("E", ctypes.c_int32), ("C", ctypes.c_int32), ("D", ctypes.c_int32)]


class _CPlanCost(ctypes.Structure):
    _fields_ = [("v_comm", ctypes.c_double), ("b_intra", ctypes.c_double), ("b_inter", ctypes.c_double),
                ("v_comp", ctypes.c_double), ("b_comp", ctypes.c_double), ("f_ckpt", ctypes.c_int32)]


@dataclass(frozen=True)
class PlanShape:
    N: int  # devices
    E: int  # experts
    C: int  # expert slots per device
    D: int  # devices per node

    def c(self) -> _CPlanShape:
        return _CPlanShape(self.N, self.E, self.C, self.D)


@dataclass(frozen=True)
class PlanCost:
    v_comm: float
    b_intra: float
    b_inter: float
    v_comp: float
    b_comp: float
    f_ckpt: int = 0

    def c(self) -> _CPlanCost:
        return _CPlanCost(self.v_comm, self.b_intra, self.b_inter, self.v_comp, self.b_comp, self.f_ckpt)


def _check(status: int, who: str):
    if status != 0:
        L = lib()
        raise MoeError(f"{who}: {L.moe_status_string(status).decode()} - {L.moe_last_error().decode()}")


def _arr(a, dtype, shape, name: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if a.shape != tuple(shape):
        raise MoeError(f"{name} has shape {a.shape}, expected {tuple(shape)}")
    return a


def _p(a: Optional[np.ndarray]):
    return ctypes.c_void_p(0) if a is None else a.ctypes.data_as(ctypes.c_void_p)


def moe_plan_replica_allocation(s: PlanShape, R) -> np.ndarray:
    R = _arr(R, np.int64, (s.N, s.E), "R")
    rep = np.empty(s.E, np.int32)
    cs = s.c()
    _check(lib().moe_plan_replica_allocation(ctypes.byref(cs), _p(R), _p(rep)), "moe_plan_replica_allocation")
    return rep


def moe_plan_expert_relocation(s: PlanShape, expert_rep, expert_loads) -> np.ndarray:
    rep = _arr(expert_rep, np.int32, (s.E,), "expert_rep")
    loads = _arr(expert_loads, np.int64, (s.E,), "expert_loads")
    A = np.empty((s.N, s.E), np.int32)
    cs = s.c()
    _check(lib().moe_plan_expert_relocation(ctypes.byref(cs), _p(rep), _p(loads), _p(A)), "moe_plan_expert_relocation")
    return A


def moe_plan_lite_routing(s: PlanShape, R, A) -> np.ndarray:
    R = _arr(R, np.int64, (s.N, s.E), "R")
    A = _arr(A, np.int32, (s.N, s.E), "A")
    S = np.empty((s.N, s.E, s.N), np.int64)
    cs = s.c()
    _check(lib().moe_plan_lite_routing(ctypes.byref(cs), _p(R), _p(A), _p(S)), "moe_plan_lite_routing")
    return S


def moe_plan_time_cost(s: PlanShape, c: PlanCost, S) -> Tuple[float, float, float]:
    S = _arr(S, np.int64, (s.N, s.E, s.N), "S")
    T = np.empty(3, np.float64)
    cs, cc = s.c(), c.c()
    _check(lib().moe_plan_time_cost(ctypes.byref(cs), ctypes.byref(cc), _p(S), _p(T)), "moe_plan_time_cost")
    return float(T[0]), float(T[1]), float(T[2])


def moe_plan_expert_layout(s: PlanShape, c: PlanCost, R, eps: int, seed: int, want_candidates: bool = False):
    """Returns (A, T, best_index[, replicas_set])."""
    R = _arr(R, np.int64, (s.N, s.E), "R")
    A = np.empty((s.N, s.E), np.int32)
    T = ctypes.c_double(0.0)
    best = ctypes.c_int32(-1)
    cands = np.empty((max(eps, 1), s.E), np.int32) if want_candidates else None
    cs, cc = s.c(), c.c()
    _check(lib().moe_plan_expert_layout(ctypes.byref(cs), ctypes.byref(cc), _p(R), ctypes.c_int32(eps),
                                        ctypes.c_uint64(seed), _p(A), ctypes.byref(T), ctypes.byref(best), _p(cands)),
           "moe_plan_expert_layout")
    if want_candidates:
        return A, T.value, best.value, cands
    return A, T.value, best.value


def moe_plan_dispatch_table(s: PlanShape, A, rank: int):
    """Returns (G, expert_of_group[G], device_of_group[G], rep_begin[E+1], rep_group[n_rep]) as numpy int32."""
    A = _arr(A, np.int32, (s.N, s.E), "A")
    cap = s.N * s.C
    eog, dog = np.empty(cap, np.int32), np.empty(cap, np.int32)
    rb, rg = np.empty(s.E + 1, np.int32), np.empty(cap, np.int32)
    G, n_rep = ctypes.c_int32(0), ctypes.c_int32(0)
    cs = s.c()
    _check(lib().moe_plan_dispatch_table(ctypes.byref(cs), _p(A), ctypes.c_int32(rank), ctypes.byref(G),
                                         ctypes.byref(n_rep), _p(eog), _p(dog), _p(rb), _p(rg)), "moe_plan_dispatch_table")
    return G.value, eog[:G.value].copy(), dog[:G.value].copy(), rb, rg[:n_rep.value].copy()
