"""Thin Python binding of the C ABI in include/jsv.h (argument marshalling only).

Every step of the search runs in the HIP kernels of libjsv.so.  PyTorch is used
for two things: the HIP stream the work is enqueued on and, optionally, the
device buffer lent to the library as workspace.  There is no CPU fallback: if
libjsv.so has not been built the import of the library fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# JSV_LIBRARY: a differently built copy of the same sources (the host-sanitizer test's build)
LIB_PATH = os.environ.get("JSV_LIBRARY") or os.path.join(_HERE, "libjsv.so")

MAX_TASKS = 16
OK, E_NULL, E_BADARG, E_CYCLE, E_OVERFLOW, E_STATE, E_WORKSPACE, E_DEVICE, E_INTERNAL = 0, -1, -2, -3, -4, -5, -6, -7, -8

EXPORTS = ["jsv_create", "jsv_destroy", "jsv_last_hip_error", "jsv_error_string", "jsv_set_objective", "jsv_set_search_space", "jsv_set_factors", "jsv_set_mixtures", "jsv_set_bounds", "jsv_set_geometry", "jsv_set_graph_mode",
           "jsv_workspace_bytes", "jsv_set_workspace", "jsv_load_profile", "jsv_set_dag",
           "jsv_search", "jsv_search_static", "jsv_eval_candidates", "jsv_get_pruned", "jsv_load_batch",
           "jsv_search_loaded_batch", "jsv_search_batch"]


class JsvResult(C.Structure):
    _fields_ = [("index", C.c_uint64), ("full_index", C.c_uint64), ("evaluated", C.c_uint64),
                ("accuracy", C.c_double), ("latency_us", C.c_uint32), ("cost_units", C.c_int32),
                ("feasible", C.c_uint32), ("flags", C.c_uint32),
                ("choice", C.c_uint16 * MAX_TASKS), ("replicas", C.c_uint32 * MAX_TASKS),
                ("objective", C.c_double),
                ("choice2", C.c_uint16 * MAX_TASKS), ("replicas2", C.c_uint32 * MAX_TASKS)]


class JsvSummary(C.Structure):
    _fields_ = [("best_level", C.c_int32), ("max_demand_mrps", C.c_uint32),
                ("seconds_device", C.c_double), ("seconds_enumerate", C.c_double),
                ("candidates_visited", C.c_uint64)]


class JsvProblem(C.Structure):
    _fields_ = [("T", C.c_uint32), ("V", C.c_uint32), ("P", C.c_uint32), ("B", C.c_uint32),
                ("units", C.c_void_p), ("batch", C.c_void_p), ("latency_us", C.c_void_p),
                ("thr_mrps", C.c_void_p), ("accuracy", C.c_void_p),
                ("E", C.c_uint32), ("src", C.c_void_p), ("dst", C.c_void_p),
                ("demand_mult_milli", C.c_void_p),
                ("capacity_units", C.c_uint32), ("queue_factor", C.c_uint32),
                ("demand_mrps", C.c_uint32), ("slo_latency_us", C.c_uint32),
                ("slo_accuracy", C.c_double), ("prune_cap", C.c_uint32)]


_lib = None


def load_library():
    """Load libjsv.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2603_08797_amd.build` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    vp, u32, f64 = C.c_void_p, C.c_uint32, C.c_double
    lib.jsv_create.restype = C.c_int
    lib.jsv_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.jsv_destroy.restype = None
    lib.jsv_destroy.argtypes = [vp]
    lib.jsv_last_hip_error.restype = C.c_int
    lib.jsv_last_hip_error.argtypes = [vp]
    lib.jsv_error_string.restype = C.c_char_p
    lib.jsv_error_string.argtypes = [C.c_int]
    lib.jsv_set_objective.restype = C.c_int
    lib.jsv_set_objective.argtypes = [vp, C.c_int, f64, f64]
    lib.jsv_set_search_space.restype = C.c_int
    lib.jsv_set_search_space.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.jsv_set_bounds.restype = C.c_int
    lib.jsv_set_bounds.argtypes = [vp, C.c_int]
    lib.jsv_set_geometry.restype = C.c_int
    lib.jsv_set_geometry.argtypes = [vp, C.c_int, C.c_int]
    lib.jsv_set_mixtures.restype = C.c_int
    lib.jsv_set_mixtures.argtypes = [vp, C.c_int]
    lib.jsv_set_factors.restype = C.c_int
    lib.jsv_set_factors.argtypes = [vp, vp]
    lib.jsv_set_graph_mode.restype = C.c_int
    lib.jsv_set_graph_mode.argtypes = [vp, C.c_int]
    lib.jsv_workspace_bytes.restype = C.c_size_t
    lib.jsv_workspace_bytes.argtypes = [vp, u32, u32]
    lib.jsv_set_workspace.restype = C.c_int
    lib.jsv_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.jsv_load_profile.restype = C.c_int
    lib.jsv_load_profile.argtypes = [vp, u32, u32, u32, u32, vp, vp, vp, vp, vp]
    lib.jsv_set_dag.restype = C.c_int
    lib.jsv_set_dag.argtypes = [vp, u32, u32, vp, vp, vp, u32, u32]
    lib.jsv_search.restype = C.c_int
    lib.jsv_search.argtypes = [vp, vp, u32, u32, f64, u32, C.POINTER(JsvResult), C.POINTER(JsvSummary)]
    lib.jsv_search_static.restype = C.c_int
    lib.jsv_search_static.argtypes = [vp, vp, u32, u32, f64, u32, C.POINTER(JsvResult), C.POINTER(JsvSummary)]
    lib.jsv_eval_candidates.restype = C.c_int
    lib.jsv_eval_candidates.argtypes = [vp, u32, u32, f64, u32, vp, u32, vp, vp, vp, vp, vp]
    lib.jsv_get_pruned.restype = C.c_int
    lib.jsv_get_pruned.argtypes = [vp, u32, u32, u32, u32, vp, C.POINTER(u32), C.POINTER(u32)]
    lib.jsv_load_batch.restype = C.c_int
    lib.jsv_load_batch.argtypes = [vp, C.POINTER(JsvProblem), u32, C.POINTER(u32)]
    lib.jsv_search_loaded_batch.restype = C.c_int
    lib.jsv_search_loaded_batch.argtypes = [vp, C.POINTER(JsvResult), C.POINTER(JsvSummary)]
    lib.jsv_search_batch.restype = C.c_int
    lib.jsv_search_batch.argtypes = [vp, C.POINTER(JsvProblem), u32, C.POINTER(JsvResult)]
    _lib = lib
    return lib


class JsvError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        msg = load_library().jsv_error_string(code).decode()
        super().__init__(f"{where}: {msg} (code {code}" + (f", hip error {hip})" if hip else ")"))
        self.code = code
        self.hip = hip


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
    choice2: List[int] = None       # mixture mode: second tuple per task (0xFFFF = none)
    replicas2: List[int] = None


@dataclass
class Summary:
    best_level: int
    max_demand_mrps: int
    seconds_device: float
    seconds_enumerate: float
    candidates_visited: int = 0


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# the same record as a numpy dtype: whole result arrays convert in one call
_RESULT_DTYPE = np.dtype([("index", "<u8"), ("full_index", "<u8"), ("evaluated", "<u8"), ("accuracy", "<f8"),
                          ("latency_us", "<u4"), ("cost_units", "<i4"), ("feasible", "<u4"), ("flags", "<u4"),
                          ("choice", "<u2", (MAX_TASKS,)), ("replicas", "<u4", (MAX_TASKS,)), ("objective", "<f8"),
                          ("choice2", "<u2", (MAX_TASKS,)), ("replicas2", "<u4", (MAX_TASKS,))])
assert _RESULT_DTYPE.itemsize == C.sizeof(JsvResult)


def _results(res, n: int, Ts) -> List[Result]:
    """n records of a JsvResult array (or of the record array that raw=True returns) as Result
    objects; Ts: tasks per record (int or list)."""
    rows = (res[:n] if isinstance(res, np.ndarray) else np.frombuffer(res, dtype=_RESULT_DTYPE, count=n)).tolist()
    out = []
    for k, (index, full, ev, acc, lat, cost, feas, flags, ch, rep, obj, ch2, rep2) in enumerate(rows):
        T = Ts if isinstance(Ts, int) else Ts[k]
        out.append(Result(index, full, ev, acc, lat, cost, bool(feas), flags, ch[:T].tolist(), rep[:T].tolist(), obj,
                          ch2[:T].tolist(), rep2[:T].tolist()))
    return out


class Jsv:
    """One search context on one GPU.

    stream: a torch.cuda.Stream (or None for torch's current stream when torch
    sees a GPU, else the default stream).  device < 0 skips every torch call,
    which is how the host-side validation is exercised on a machine without a GPU.
    """

    def __init__(self, device: int = 0, stream=None, use_torch: bool = True):
        self._torch = None
        handle = None
        if use_torch:
            # torch first: the library must bind to the HIP runtime torch has loaded, so that
            # streams and device pointers of both live in one runtime
            import torch
        self._lib = load_library()
        if use_torch:
            if torch.cuda.is_available():
                self._torch = torch
                s = stream if stream is not None else torch.cuda.current_stream(device)
                self._stream = s                      # keep it alive
                handle = C.c_void_p(s.cuda_stream)
        h = C.c_void_p()
        rc = self._lib.jsv_create(C.byref(h), int(device), handle)
        if rc != OK:
            raise JsvError(rc, "jsv_create")
        self._h = h
        self._ws = None
        self.T = 0
        self.C = 0
        self._batch_T: List[int] = []

    def close(self):
        if getattr(self, "_h", None):
            self._lib.jsv_destroy(self._h)
            self._h = None
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, where: str):
        if rc != OK:
            raise JsvError(rc, where, self._lib.jsv_last_hip_error(self._h))

    def set_objective(self, mode: int, alpha: float = 1.0, beta: float = 0.035):
        """mode 0: cheapest feasible; mode 1: maximise alpha*A_obj - beta*cost (Eq. 14)."""
        self._check(self._lib.jsv_set_objective(self._h, int(mode), float(alpha), float(beta)),
                    "jsv_set_objective")

    def set_search_space(self, accuracy_scaling=True, spatial_partitioning=True, graph_informed=True):
        """Restrictions of the paper's ablations (A, S, T); all on by default."""
        self._check(self._lib.jsv_set_search_space(self._h, int(accuracy_scaling), int(spatial_partitioning),
                                                   int(graph_informed)), "jsv_set_search_space")

    def set_factors(self, factor_milli):
        """Per-variant multiplicative factors (Eq. 4, 5), [E][V] in 1/1000ths in the edge order of
        set_dag; None returns to the fixed multipliers.  Call after load_profile and set_dag."""
        if factor_milli is None:
            self._check(self._lib.jsv_set_factors(self._h, None), "jsv_set_factors")
            return
        f = _u32(factor_milli)
        if f.shape != (getattr(self, "E", -1), getattr(self, "V", -1)):
            raise ValueError("factor_milli must have shape [E][V] of the loaded graph and profile")
        self._check(self._lib.jsv_set_factors(self._h, f.ctypes.data_as(C.c_void_p)), "jsv_set_factors")

    def set_bounds(self, on: bool = True):
        """Skip candidates that latency or capacity bounds exclude in bulk (default on); the
        result does not depend on it."""
        self._check(self._lib.jsv_set_bounds(self._h, int(on)), "jsv_set_bounds")

    def set_geometry(self, blocks_per_cu: int = 0, lanes_percent: int = 0):
        """Launch geometry of the enumeration (0 = automatic); the result does not depend on it."""
        self._check(self._lib.jsv_set_geometry(self._h, int(blocks_per_cu), int(lanes_percent)), "jsv_set_geometry")

    def set_mixtures(self, on: bool = True):
        """Let a task run two tuples side by side (Eq. 2, 6, 7, 9, 10)."""
        self._check(self._lib.jsv_set_mixtures(self._h, int(on)), "jsv_set_mixtures")

    def set_graph_mode(self, on: bool = True):
        """Record the launch sequence of a search into a HIP graph and replay it."""
        self._check(self._lib.jsv_set_graph_mode(self._h, int(on)), "jsv_set_graph_mode")

    # -- inputs ------------------------------------------------------------------
    def load_profile(self, T, V, P, B, units, batch, latency_us, thr_mrps, accuracy):
        u, b, l = _u32(units), _u32(batch), _u32(latency_us)
        h = None if thr_mrps is None else _u32(thr_mrps)
        a = np.ascontiguousarray(accuracy, dtype=np.float64)
        self._check(self._lib.jsv_load_profile(self._h, int(T), int(V), int(P), int(B), _ptr(u),
                                               _ptr(b), _ptr(l), _ptr(h), _ptr(a)), "jsv_load_profile")
        self.T, self.C, self.V = int(T), int(V) * int(P) * int(B), int(V)

    def set_dag(self, T, src, dst, demand_mult_milli, capacity_units, queue_factor=2):
        s = np.ascontiguousarray(src, dtype=np.uint16)
        d = np.ascontiguousarray(dst, dtype=np.uint16)
        m = _u32(demand_mult_milli)
        self._check(self._lib.jsv_set_dag(self._h, int(T), int(s.shape[0]), _ptr(s), _ptr(d), _ptr(m),
                                          int(capacity_units), int(queue_factor)), "jsv_set_dag")
        self.E = int(s.shape[0])

    def load(self, pb, derive_throughput: bool = False):
        """Profile and graph of a workloads.Problem."""
        self.load_profile(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us,
                          None if derive_throughput else pb.thr_mrps, pb.accuracy)
        self.set_dag(pb.T, pb.src, pb.dst, pb.mult_milli, pb.capacity_units, pb.queue_factor)

    # -- workspace -----------------------------------------------------------------
    def workspace_bytes(self, n_levels: int, prune_cap: int) -> int:
        return int(self._lib.jsv_workspace_bytes(self._h, int(n_levels), int(prune_cap)))

    def lend_workspace(self, n_levels: int, prune_cap: int):
        """Allocate the workspace as a torch tensor and lend it to the library."""
        if self._torch is None:
            raise RuntimeError("no GPU visible to torch")
        n = self.workspace_bytes(n_levels, prune_cap)
        t = self._torch.empty(n + 256, dtype=self._torch.uint8, device="cuda")
        p = (t.data_ptr() + 255) // 256 * 256
        self._check(self._lib.jsv_set_workspace(self._h, C.c_void_p(p), n), "jsv_set_workspace")
        self._ws = t
        return n

    # -- search ----------------------------------------------------------------------
    def search(self, demand_mrps, slo_latency_us: int, slo_accuracy: float, prune_cap: int = 0, raw: bool = False):
        """raw=True: the records as the library wrote them (a numpy record array over the C structs,
        one per level; `results()` turns it into Result objects) instead of a list of Result."""
        d = _u32(demand_mrps)
        n = int(d.shape[0])
        res = (JsvResult * max(n, 1))()
        summ = JsvSummary()
        self._check(self._lib.jsv_search(self._h, _ptr(d), n, int(slo_latency_us), float(slo_accuracy),
                                         int(prune_cap), res, C.byref(summ)), "jsv_search")
        return (np.frombuffer(res, dtype=_RESULT_DTYPE, count=n) if raw else _results(res, n, self.T),
                Summary(int(summ.best_level), int(summ.max_demand_mrps), float(summ.seconds_device),
                        float(summ.seconds_enumerate), int(summ.candidates_visited)))

    def search_static(self, demand_mrps, slo_latency_us: int, slo_accuracy: float, prune_cap: int = 0):
        """jsv_search without any allocation: everything lives in the library's static device array."""
        d = _u32(demand_mrps)
        n = int(d.shape[0])
        res = (JsvResult * max(n, 1))()
        summ = JsvSummary()
        self._check(self._lib.jsv_search_static(self._h, _ptr(d), n, int(slo_latency_us), float(slo_accuracy),
                                                int(prune_cap), res, C.byref(summ)), "jsv_search_static")
        return (_results(res, n, self.T),
                Summary(int(summ.best_level), int(summ.max_demand_mrps), float(summ.seconds_device),
                        float(summ.seconds_enumerate), int(summ.candidates_visited)))

    def eval_candidates(self, demand_mrps: int, slo_latency_us: int, slo_accuracy: float,
                        prune_cap: int, index):
        idx = np.ascontiguousarray(index, dtype=np.uint64)
        n = int(idx.shape[0])
        lat = np.zeros(n, dtype=np.uint32)
        rep = np.zeros((n, self.T), dtype=np.uint32)
        cost = np.zeros(n, dtype=np.int32)
        acc = np.zeros(n, dtype=np.float64)
        mask = np.zeros(n, dtype=np.uint8)
        self._check(self._lib.jsv_eval_candidates(self._h, int(demand_mrps), int(slo_latency_us),
                                                  float(slo_accuracy), int(prune_cap), _ptr(idx), n,
                                                  _ptr(lat), _ptr(rep), _ptr(cost), _ptr(acc), _ptr(mask)),
                    "jsv_eval_candidates")
        return lat, rep, cost, acc, mask

    def get_pruned(self, demand_mrps: int, slo_latency_us: int, prune_cap: int, task: int):
        ids = np.zeros(max(self.C, 1), dtype=np.uint16)
        K, tr = C.c_uint32(), C.c_uint32()
        self._check(self._lib.jsv_get_pruned(self._h, int(demand_mrps), int(slo_latency_us),
                                             int(prune_cap), int(task), _ptr(ids), C.byref(K), C.byref(tr)),
                    "jsv_get_pruned")
        return ids[:K.value].copy(), bool(tr.value)

    # -- batch -------------------------------------------------------------------------
    def _marshal_batch(self, problems, searches):
        n = len(problems)
        arr = (JsvProblem * n)()
        keep = []
        for k, (pb, se) in enumerate(zip(problems, searches)):
            bufs = [_u32(pb.units), _u32(pb.batch), _u32(pb.latency_us), _u32(pb.thr_mrps),
                    np.ascontiguousarray(pb.accuracy, dtype=np.float64),
                    np.ascontiguousarray(pb.src, dtype=np.uint16),
                    np.ascontiguousarray(pb.dst, dtype=np.uint16), _u32(pb.mult_milli)]
            keep.append(bufs)
            p = arr[k]
            p.T, p.V, p.P, p.B = pb.T, pb.V, pb.P, pb.B
            p.units, p.batch, p.latency_us, p.thr_mrps, p.accuracy = [b.ctypes.data for b in bufs[:5]]
            p.E = int(bufs[5].shape[0])
            p.src, p.dst, p.demand_mult_milli = bufs[5].ctypes.data, bufs[6].ctypes.data, bufs[7].ctypes.data
            p.capacity_units, p.queue_factor = int(pb.capacity_units), int(pb.queue_factor)
            assert len(se.demand_mrps) == 1
            p.demand_mrps = int(se.demand_mrps[0])
            p.slo_latency_us, p.slo_accuracy, p.prune_cap = int(se.slo_latency_us), float(se.slo_accuracy), int(se.prune_cap)
        return arr, keep

    def load_batch(self, problems: Sequence, searches: Sequence):
        arr, keep = self._marshal_batch(problems, searches)
        bad = C.c_uint32()
        rc = self._lib.jsv_load_batch(self._h, arr, len(problems), C.byref(bad))
        if rc != OK:
            raise JsvError(rc, f"jsv_load_batch (problem {bad.value})", self._lib.jsv_last_hip_error(self._h))
        self._batch_T = [pb.T for pb in problems]

    def results(self, records, batch: bool = False) -> List[Result]:
        """The record array of a raw=True search as Result objects."""
        return _results(records, int(records.shape[0]), self._batch_T if batch else self.T)

    def search_loaded_batch(self, raw: bool = False):
        n = len(self._batch_T)
        res = (JsvResult * max(n, 1))()
        summ = JsvSummary()
        self._check(self._lib.jsv_search_loaded_batch(self._h, res, C.byref(summ)), "jsv_search_loaded_batch")
        return (np.frombuffer(res, dtype=_RESULT_DTYPE, count=n) if raw else _results(res, n, self._batch_T),
                Summary(int(summ.best_level), int(summ.max_demand_mrps), float(summ.seconds_device),
                        float(summ.seconds_enumerate), int(summ.candidates_visited)))

    def search_batch(self, problems: Sequence, searches: Sequence):
        arr, keep = self._marshal_batch(problems, searches)
        n = len(problems)
        res = (JsvResult * max(n, 1))()
        self._check(self._lib.jsv_search_batch(self._h, arr, n, res), "jsv_search_batch")
        self._batch_T = [pb.T for pb in problems]
        return _results(res, n, self._batch_T)
