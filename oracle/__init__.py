"""ctypes front end of the CPU oracle (oracle/jsv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The library under test never imports this
package, and this package never imports the library under test.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jsv_oracle.c")
_LIB = os.path.join(_HERE, "libjsv_oracle.so")

MAX_TASKS = 16
OK, E_ARG, E_CYCLE, E_RANGE, E_MEM = 0, -1, -2, -3, -4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB, _SRC])
    return _LIB


class OrcResult(C.Structure):
    _fields_ = [("index", C.c_uint64), ("full_index", C.c_uint64), ("evaluated", C.c_uint64),
                ("accuracy", C.c_double), ("latency_us", C.c_uint32), ("cost", C.c_int32),
                ("feasible", C.c_uint32), ("flags", C.c_uint32),
                ("choice", C.c_uint16 * MAX_TASKS), ("replicas", C.c_uint32 * MAX_TASKS),
                ("objective", C.c_double),
                ("choice2", C.c_uint16 * MAX_TASKS), ("replicas2", C.c_uint32 * MAX_TASKS)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # JSV_ORACLE_LIBRARY: a differently built copy of the same source (the sanitizer test's)
        alt = os.environ.get("JSV_ORACLE_LIBRARY")
        if not alt:
            build()
        lib = C.CDLL(alt or _LIB)
        vp = C.c_void_p
        lib.orc_create.restype = C.c_int
        lib.orc_create.argtypes = [C.POINTER(vp), C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                   vp, vp, vp, vp, vp, C.c_uint32, vp, vp, vp, C.c_uint32, C.c_uint32]
        lib.orc_destroy.restype = None
        lib.orc_destroy.argtypes = [vp]
        lib.orc_num_paths.restype = C.c_int
        lib.orc_num_paths.argtypes = [vp]
        lib.orc_amax.restype = C.c_double
        lib.orc_amax.argtypes = [vp]
        lib.orc_get_path.restype = C.c_int
        lib.orc_get_path.argtypes = [vp, C.c_int, vp, C.POINTER(C.c_double)]
        lib.orc_cost_table.restype = C.c_int
        lib.orc_cost_table.argtypes = [vp, C.c_uint32, vp, vp]
        lib.orc_pruned.restype = C.c_int
        lib.orc_pruned.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, vp,
                                   C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        lib.orc_search.restype = C.c_int
        lib.orc_search.argtypes = [vp, vp, C.c_uint32, C.c_uint32, C.c_double, C.c_uint32, C.c_int,
                                   C.POINTER(OrcResult), C.POINTER(C.c_int32), C.POINTER(C.c_uint32)]
        lib.orc_search_range.restype = C.c_int
        lib.orc_search_range.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_double, C.c_uint32,
                                         C.c_uint64, C.c_uint64, C.c_int, C.POINTER(OrcResult)]
        lib.orc_space.restype = C.c_int
        lib.orc_space.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, vp,
                                  C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]
        lib.orc_eval.restype = C.c_int
        lib.orc_eval.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_double, C.c_uint32, vp, C.c_uint32,
                                 vp, vp, vp, vp, vp]
        lib.orc_accuracy_of_variants.restype = C.c_double
        lib.orc_accuracy_of_variants.argtypes = [vp, vp]
        lib.orc_accuracy_margin.restype = C.c_double
        lib.orc_accuracy_margin.argtypes = [vp, C.c_double]
        lib.orc_set_objective.restype = C.c_int
        lib.orc_set_objective.argtypes = [vp, C.c_int, C.c_double, C.c_double]
        lib.orc_objective_margin.restype = C.c_int
        lib.orc_objective_margin.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_double, C.c_uint32,
                                             C.POINTER(C.c_double)]
        lib.orc_set_search_space.restype = C.c_int
        lib.orc_set_search_space.argtypes = [vp, C.c_int, C.c_int, C.c_int]
        lib.orc_set_mixtures.restype = C.c_int
        lib.orc_set_mixtures.argtypes = [vp, C.c_int]
        lib.orc_options.restype = C.c_int
        lib.orc_options.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                    vp, vp, vp, vp, vp, vp, vp, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        lib.orc_mixture_margin.restype = C.c_int
        lib.orc_mixture_margin.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_double, C.c_uint32,
                                           C.POINTER(C.c_double)]
        lib.orc_set_factors.restype = C.c_int
        lib.orc_set_factors.argtypes = [vp, vp]
        lib.orc_budget_margin.restype = C.c_double
        lib.orc_budget_margin.argtypes = [vp]
        lib.orc_max_threads.restype = C.c_int
        lib.orc_max_threads.argtypes = []
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle: {where} failed with code {code}")
        self.code = code


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Result:
    index: int
    full_index: int
    evaluated: int
    accuracy: float
    latency_us: int
    cost: int
    feasible: bool
    flags: int
    choice: List[int]
    replicas: List[int]
    objective: float = 0.0
    choice2: List[int] = None       # mixtures: second tuple per task (0xFFFF = none)
    replicas2: List[int] = None


def _result(r: OrcResult, T: int) -> Result:
    return Result(int(r.index), int(r.full_index), int(r.evaluated), float(r.accuracy),
                  int(r.latency_us), int(r.cost), bool(r.feasible), int(r.flags),
                  [int(r.choice[t]) for t in range(T)], [int(r.replicas[t]) for t in range(T)],
                  float(r.objective), [int(r.choice2[t]) for t in range(T)],
                  [int(r.replicas2[t]) for t in range(T)])


def max_threads() -> int:
    return int(_load().orc_max_threads())


class Oracle:
    """One compound system (profile tables + task graph) held by the oracle."""

    def __init__(self, T, V, P, B, units, batch, latency_us, thr_mrps, accuracy, src, dst,
                 mult_milli, capacity_units, queue_factor=2):
        lib = _load()
        self.T, self.V, self.P, self.B = int(T), int(V), int(P), int(B)
        self.C = self.V * self.P * self.B
        self._keep = [
            np.ascontiguousarray(units, dtype=np.uint32),
            np.ascontiguousarray(batch, dtype=np.uint32),
            np.ascontiguousarray(latency_us, dtype=np.uint32),
            None if thr_mrps is None else np.ascontiguousarray(thr_mrps, dtype=np.uint32),
            np.ascontiguousarray(accuracy, dtype=np.float64),
            np.ascontiguousarray(src, dtype=np.uint16),
            np.ascontiguousarray(dst, dtype=np.uint16),
            np.ascontiguousarray(mult_milli, dtype=np.uint32),
        ]
        k = self._keep
        h = C.c_void_p()
        rc = lib.orc_create(C.byref(h), self.T, self.V, self.P, self.B, _ptr(k[0]), _ptr(k[1]),
                            _ptr(k[2]), _ptr(k[3]), _ptr(k[4]), int(k[5].shape[0]), _ptr(k[5]),
                            _ptr(k[6]), _ptr(k[7]), int(capacity_units), int(queue_factor))
        if rc != OK:
            raise OracleError(rc, "orc_create")
        self._h = h
        self._lib = lib

    @classmethod
    def from_problem(cls, pb, derive_throughput: bool = False) -> "Oracle":
        return cls(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us,
                   None if derive_throughput else pb.thr_mrps, pb.accuracy, pb.src, pb.dst,
                   pb.mult_milli, pb.capacity_units, pb.queue_factor)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_objective(self, mode: int, alpha: float = 1.0, beta: float = 0.035):
        """mode 0: cheapest feasible; mode 1: maximise alpha*A_obj - beta*cost."""
        rc = self._lib.orc_set_objective(self._h, int(mode), float(alpha), float(beta))
        if rc != OK:
            raise OracleError(rc, "orc_set_objective")

    def set_search_space(self, accuracy_scaling=True, spatial_partitioning=True, graph_informed=True):
        """Restrictions of the paper's ablations: A (variants), S (partitions), T (global budgets)."""
        rc = self._lib.orc_set_search_space(self._h, int(accuracy_scaling), int(spatial_partitioning),
                                            int(graph_informed))
        if rc != OK:
            raise OracleError(rc, "orc_set_search_space")

    def set_factors(self, factor_milli):
        """Per-variant multiplicative factors F(t, v, t') of Eq. 4, [E][V] in 1/1000ths in the
        edge order of the model; None returns to the fixed per-task multipliers."""
        if factor_milli is None:
            rc = self._lib.orc_set_factors(self._h, None)
        else:
            f = np.ascontiguousarray(factor_milli, dtype=np.uint32)
            if f.shape != (int(self._keep[5].shape[0]), self.V):
                raise ValueError("factor_milli must have shape [E][V]")
            rc = self._lib.orc_set_factors(self._h, _ptr(f))
        if rc != OK:
            raise OracleError(rc, "orc_set_factors")

    def set_mixtures(self, on: bool = True):
        """Let a task mix two tuples (Eq. 2, 6, 7, 9, 10 with two active instance types)."""
        rc = self._lib.orc_set_mixtures(self._h, int(on))
        if rc != OK:
            raise OracleError(rc, "orc_set_mixtures")

    def options(self, demand_mrps: int, slo_latency_us: int, prune_cap: int, task: int, room: int = 1 << 20):
        """Mixture mode: surviving options of one task as a list of
        (c1, c2, m1, m2, latency_us, cost, accuracy) in ascending id, and the thinning flag."""
        c1 = np.zeros(room, dtype=np.uint16); c2 = np.zeros(room, dtype=np.uint16)
        m1 = np.zeros(room, dtype=np.uint32); m2 = np.zeros(room, dtype=np.uint32)
        lat = np.zeros(room, dtype=np.uint32); cost = np.zeros(room, dtype=np.int32)
        acc = np.zeros(room, dtype=np.float64)
        n, tr = C.c_uint32(), C.c_uint32()
        rc = self._lib.orc_options(self._h, int(demand_mrps), int(slo_latency_us), int(prune_cap), int(task),
                                   room, _ptr(c1), _ptr(c2), _ptr(m1), _ptr(m2), _ptr(lat), _ptr(cost), _ptr(acc),
                                   C.byref(n), C.byref(tr))
        if rc != OK:
            raise OracleError(rc, "orc_options")
        if n.value > room:
            raise OracleError(ORC_E_RANGE if "ORC_E_RANGE" in globals() else -3, "orc_options: room")
        k = n.value
        return [(int(c1[i]), int(c2[i]), int(m1[i]), int(m2[i]), int(lat[i]), int(cost[i]), float(acc[i]))
                for i in range(k)], bool(tr.value)

    def mixture_margin(self, demand_mrps: int, slo_latency_us: int, slo_accuracy: float, prune_cap: int) -> float:
        m = C.c_double()
        rc = self._lib.orc_mixture_margin(self._h, int(demand_mrps), int(slo_latency_us), float(slo_accuracy),
                                          int(prune_cap), C.byref(m))
        if rc != OK:
            raise OracleError(rc, "orc_mixture_margin")
        return float(m.value)

    def budget_margin(self) -> float:
        return float(self._lib.orc_budget_margin(self._h))

    def objective_margin(self, demand_mrps: int, slo_latency_us: int, slo_accuracy: float,
                         prune_cap: int) -> float:
        m = C.c_double()
        rc = self._lib.orc_objective_margin(self._h, int(demand_mrps), int(slo_latency_us),
                                            float(slo_accuracy), int(prune_cap), C.byref(m))
        if rc != OK:
            raise OracleError(rc, "orc_objective_margin")
        return float(m.value)

    # -- graph -----------------------------------------------------------------
    def amax(self) -> float:
        return float(self._lib.orc_amax(self._h))

    def paths(self) -> List[Tuple[List[int], float]]:
        out = []
        nodes = np.zeros(self.T, dtype=np.int32)
        f = C.c_double()
        for k in range(self._lib.orc_num_paths(self._h)):
            n = self._lib.orc_get_path(self._h, k, _ptr(nodes), C.byref(f))
            out.append(([int(x) for x in nodes[:n]], float(f.value)))
        return out

    def accuracy_of_variants(self, variants: Sequence[int]) -> float:
        v = np.ascontiguousarray(variants, dtype=np.uint32)
        assert v.shape[0] == self.T
        return float(self._lib.orc_accuracy_of_variants(self._h, _ptr(v)))

    # -- per level ---------------------------------------------------------------
    def cost_table(self, demand_mrps: int):
        rep = np.zeros((self.T, self.C), dtype=np.uint32)
        cost = np.zeros((self.T, self.C), dtype=np.int32)
        rc = self._lib.orc_cost_table(self._h, int(demand_mrps), _ptr(rep), _ptr(cost))
        if rc != OK:
            raise OracleError(rc, "orc_cost_table")
        return rep, cost

    def pruned(self, demand_mrps: int, slo_latency_us: int, prune_cap: int, task: int):
        ids = np.zeros(self.C, dtype=np.uint16)
        K, tr = C.c_uint32(), C.c_uint32()
        rc = self._lib.orc_pruned(self._h, int(demand_mrps), int(slo_latency_us), int(prune_cap),
                                  int(task), _ptr(ids), C.byref(K), C.byref(tr))
        if rc != OK:
            raise OracleError(rc, "orc_pruned")
        return ids[:K.value].copy(), bool(tr.value)

    def space(self, demand_mrps: int, slo_latency_us: int, prune_cap: int):
        K = np.zeros(self.T, dtype=np.uint32)
        n, tr = C.c_uint64(), C.c_uint32()
        rc = self._lib.orc_space(self._h, int(demand_mrps), int(slo_latency_us), int(prune_cap),
                                 _ptr(K), C.byref(n), C.byref(tr))
        if rc != OK:
            raise OracleError(rc, "orc_space")
        return K, int(n.value), bool(tr.value)

    def search(self, demand_mrps, slo_latency_us: int, slo_accuracy: float, prune_cap: int = 0,
               threads: int = 1):
        d = np.ascontiguousarray(demand_mrps, dtype=np.uint32)
        n = int(d.shape[0])
        res = (OrcResult * n)()
        bl, md = C.c_int32(), C.c_uint32()
        rc = self._lib.orc_search(self._h, _ptr(d), n, int(slo_latency_us), float(slo_accuracy),
                                  int(prune_cap), int(threads), res, C.byref(bl), C.byref(md))
        if rc != OK:
            raise OracleError(rc, "orc_search")
        return [_result(res[i], self.T) for i in range(n)], int(bl.value), int(md.value)

    def search_range(self, demand_mrps: int, slo_latency_us: int, slo_accuracy: float,
                     prune_cap: int, lo: int, hi: int, threads: int = 1) -> Result:
        res = OrcResult()
        rc = self._lib.orc_search_range(self._h, int(demand_mrps), int(slo_latency_us),
                                        float(slo_accuracy), int(prune_cap), int(lo), int(hi),
                                        int(threads), C.byref(res))
        if rc != OK:
            raise OracleError(rc, "orc_search_range")
        return _result(res, self.T)

    def eval(self, demand_mrps: int, slo_latency_us: int, slo_accuracy: float, prune_cap: int,
             index):
        idx = np.ascontiguousarray(index, dtype=np.uint64)
        n = int(idx.shape[0])
        lat = np.zeros(n, dtype=np.uint32)
        rep = np.zeros((n, self.T), dtype=np.uint32)
        cost = np.zeros(n, dtype=np.int32)
        acc = np.zeros(n, dtype=np.float64)
        mask = np.zeros(n, dtype=np.uint8)
        rc = self._lib.orc_eval(self._h, int(demand_mrps), int(slo_latency_us), float(slo_accuracy),
                                int(prune_cap), _ptr(idx), n, _ptr(lat), _ptr(rep), _ptr(cost),
                                _ptr(acc), _ptr(mask))
        if rc != OK:
            raise OracleError(rc, "orc_eval")
        return lat, rep, cost, acc, mask

    # -- input guard band ---------------------------------------------------------
    def accuracy_margin(self, slo_accuracy: float) -> float:
        """Smallest |A_obj - SLO_a| over every combination of variants."""
        return float(self._lib.orc_accuracy_margin(self._h, float(slo_accuracy)))
