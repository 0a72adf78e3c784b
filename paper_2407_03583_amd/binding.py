"""Thin ctypes binding of libloki_alloc.so (include/loki_alloc.h).

Argument marshalling only: every step of the search runs in the library's
kernels.  PyTorch supplies the device workspace and the stream, nothing else.
There is no CPU fallback: if the library or a GPU is missing, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libloki_alloc.so")

MAX_TASKS = 8
MAX_VARIANTS = 8

LOKI_OK = 0
LOKI_E_NULL, LOKI_E_INVALID_GRAPH, LOKI_E_RANGE, LOKI_E_WORKSPACE, LOKI_E_HIP, LOKI_E_ARG = -1, -2, -3, -4, -5, -6
LOKI_E_STATIC_LIMIT = -7
LOKI_STATIC_SCRATCH_BYTES, LOKI_STATIC_MAX_DEMAND_POINTS = 4 << 20, 64
LOKI_TIE_WORKERS_THEN_INDEX, LOKI_TIE_INDEX_ONLY, LOKI_SEARCH_PER_LANE = 0, 1, 2
LOKI_FOUND, LOKI_NO_FEASIBLE = 0, 1
LOKI_BAD_WORKERS, LOKI_BAD_DEMAND, LOKI_BAD_EMPTY, LOKI_BAD_LATENCY = 1, 2, 4, 8
LOKI_PHASE_HARDWARE, LOKI_PHASE_ACCURACY, LOKI_PHASE_OVERLOAD = 0, 1, 2
UINT64_MAX = (1 << 64) - 1

EXPORTS = ["loki_problem_create", "loki_problem_destroy", "loki_num_candidates", "loki_workspace_bytes",
           "loki_decode", "loki_alloc_search", "loki_alloc_search_enqueue", "loki_alloc_search_static", "loki_alloc_eval",
           "loki_route_table", "loki_route_workspace_bytes", "loki_route_table_batch", "loki_plan_trace", "loki_last_search_ms", "loki_last_search_plans_scored", "loki_last_search_fill_bits", "loki_strerror", "loki_last_hip_error"]


class LokiError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().loki_strerror(code).decode()
        if code == LOKI_E_HIP:
            msg += f" (hipError {lib().loki_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


class PipelineC(C.Structure):
    _fields_ = [("n_tasks", C.c_int32),
                ("parent", C.POINTER(C.c_int32)),
                ("fanout_q4", C.POINTER(C.c_int32)),
                ("n_variants", C.POINTER(C.c_int32)),
                ("n_batches", C.POINTER(C.c_int32)),
                ("batch_size", C.POINTER(C.c_int32)),
                ("max_replicas", C.POINTER(C.c_int32)),
                ("acc_ppm", C.POINTER(C.c_int32)),
                ("latency_us", C.POINTER(C.c_int64)),
                ("thr_mqps", C.POINTER(C.c_int64)),
                ("variant_factor_q4", C.POINTER(C.c_int32)),
                ("per_variant_batch", C.c_int32),
                ("path_acc_ppm", C.POINTER(C.c_int32)),
                ("latency_per_path", C.c_int32)]


class Result(C.Structure):
    _fields_ = [("index", C.c_uint64),
                ("accuracy", C.c_double),
                ("n_feasible", C.c_uint64),
                ("workers_used", C.c_int32),
                ("status", C.c_int32)]

    def as_tuple(self):
        """(index, accuracy, n_feasible, workers, found) -- found = 1 when a plan was returned."""
        return (int(self.index), float(self.accuracy), int(self.n_feasible), int(self.workers_used),
                1 if self.status == LOKI_FOUND else 0)


class PlanStep(C.Structure):
    _fields_ = [("estimate_mqps", C.c_int64),
                ("plan", Result),
                ("phase", C.c_int32),
                ("pad", C.c_int32)]


class Eval(C.Structure):
    _fields_ = [("accuracy", C.c_double),
                ("workers", C.c_int32),
                ("infeasible", C.c_uint32)]


class Route(C.Structure):
    _fields_ = [("demand", C.c_int64 * MAX_TASKS),
                ("scale", C.c_int64 * MAX_TASKS),
                ("unserved", C.c_int64 * MAX_TASKS),
                ("replicas", (C.c_int32 * MAX_VARIANTS) * MAX_TASKS),
                ("batch", (C.c_int32 * MAX_VARIANTS) * MAX_TASKS),
                ("capacity", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("routed", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("leftover", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("budget_us", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("prob", ((C.c_double * MAX_VARIANTS) * MAX_VARIANTS) * MAX_TASKS)]


_lib = None


def lib():
    """Load the in-tree library (build it first with paper_2407_03583_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2407_03583_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        # PyTorch owns the device memory and the stream this library works on, so its HIP runtime
        # must be the one in the process: load it before the library pulls in another copy.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        P = C.c_void_p
        L.loki_problem_create.restype = C.c_int
        L.loki_problem_create.argtypes = [C.POINTER(PipelineC), C.POINTER(P)]
        L.loki_problem_destroy.restype = None
        L.loki_problem_destroy.argtypes = [P]
        L.loki_num_candidates.restype = C.c_int
        L.loki_num_candidates.argtypes = [P, C.POINTER(C.c_uint64)]
        L.loki_workspace_bytes.restype = C.c_int
        L.loki_workspace_bytes.argtypes = [P, C.c_int64, C.POINTER(C.c_size_t)]
        L.loki_decode.restype = C.c_int
        L.loki_decode.argtypes = [P, C.c_uint64, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        search_args = [P, C.POINTER(C.c_int64), C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_uint32,
                       C.c_uint64, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]
        L.loki_alloc_search.restype = C.c_int
        L.loki_alloc_search.argtypes = search_args + [C.POINTER(Result)]
        L.loki_alloc_search_enqueue.restype = C.c_int
        L.loki_alloc_search_enqueue.argtypes = search_args + [C.c_void_p]
        L.loki_alloc_search_static.restype = C.c_int
        L.loki_alloc_search_static.argtypes = search_args[:9] + [C.c_void_p, C.POINTER(Result)]
        L.loki_alloc_eval.restype = C.c_int
        L.loki_alloc_eval.argtypes = [P, C.POINTER(C.c_uint64), C.c_int64, C.c_int64, C.c_int32, C.c_int64,
                                      C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(Eval)]
        L.loki_route_table.restype = C.c_int
        L.loki_route_table.argtypes = [P, C.c_uint64, C.c_int64, C.POINTER(Route)]
        L.loki_route_workspace_bytes.restype = C.c_int
        L.loki_route_workspace_bytes.argtypes = [P, C.c_int64, C.POINTER(C.c_size_t)]
        L.loki_route_table_batch.restype = C.c_int
        L.loki_route_table_batch.argtypes = [P, C.POINTER(C.c_uint64), C.POINTER(C.c_int64), C.c_int64, C.c_void_p,
                                             C.c_size_t, C.c_void_p, C.POINTER(Route)]
        L.loki_plan_trace.restype = C.c_int
        L.loki_plan_trace.argtypes = [P, C.POINTER(C.c_int64), C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                      C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(PlanStep)]
        L.loki_last_search_ms.restype = C.c_int
        L.loki_last_search_ms.argtypes = [P, C.POINTER(C.c_float)]
        L.loki_last_search_plans_scored.restype = C.c_int
        L.loki_last_search_plans_scored.argtypes = [P, C.POINTER(C.c_uint64)]
        L.loki_last_search_fill_bits.restype = C.c_int
        L.loki_last_search_fill_bits.argtypes = [P, C.POINTER(C.c_int32)]
        L.loki_strerror.restype = C.c_char_p
        L.loki_strerror.argtypes = [C.c_int]
        L.loki_last_hip_error.restype = C.c_int
        L.loki_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _check(code: int, where: str):
    if code != LOKI_OK:
        raise LokiError(code, where)


def _arr(ctype, values: Sequence[int]):
    return (ctype * max(1, len(values)))(*[int(v) for v in values])


def _pipeline_struct(p):
    keep = [_arr(C.c_int32, p.parent), _arr(C.c_int32, p.fanout_q4), _arr(C.c_int32, p.n_variants),
            _arr(C.c_int32, p.n_batches), _arr(C.c_int32, p.batch_size), _arr(C.c_int32, p.max_replicas),
            _arr(C.c_int32, p.acc_ppm), _arr(C.c_int64, p.latency_us), _arr(C.c_int64, p.thr_mqps)]
    vf = getattr(p, "variant_factor_q4", None)
    vf_arr = _arr(C.c_int32, vf) if vf is not None else None
    pt = getattr(p, "path_acc_ppm", None)
    pt_arr = _arr(C.c_int32, pt) if pt is not None else None
    s = PipelineC(int(p.n_tasks), *[C.cast(a, C.POINTER(a._type_)) for a in keep],
                  C.cast(vf_arr, C.POINTER(C.c_int32)) if vf_arr is not None else C.POINTER(C.c_int32)(),
                  1 if getattr(p, "per_variant_batch", False) else 0,
                  C.cast(pt_arr, C.POINTER(C.c_int32)) if pt_arr is not None else C.POINTER(C.c_int32)(),
                  1 if getattr(p, "latency_per_path", False) else 0)
    keep.extend([vf_arr, pt_arr])
    return s, keep


class Problem:
    """A loki_problem_t handle plus a torch-owned device workspace."""

    def __init__(self, pipeline):
        self._h = C.c_void_p()
        s, keep = _pipeline_struct(pipeline)
        _check(lib().loki_problem_create(C.byref(s), C.byref(self._h)), "loki_problem_create")
        self.n_tasks = int(pipeline.n_tasks)
        self.n_variants = [int(v) for v in pipeline.n_variants]
        self.per_variant_batch = bool(getattr(pipeline, "per_variant_batch", False))
        self._ws = None

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().loki_problem_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def num_candidates(self) -> int:
        n = C.c_uint64()
        _check(lib().loki_num_candidates(self._h, C.byref(n)), "loki_num_candidates")
        return int(n.value)

    def workspace_bytes(self, n_demand: int) -> int:
        b = C.c_size_t()
        _check(lib().loki_workspace_bytes(self._h, n_demand, C.byref(b)), "loki_workspace_bytes")
        return int(b.value)

    def decode(self, index: int):
        x = (C.c_int32 * sum(self.n_variants))()
        b = (C.c_int32 * (sum(self.n_variants) if self.per_variant_batch else self.n_tasks))()
        _check(lib().loki_decode(self._h, index, x, b), "loki_decode")
        return list(x), list(b)

    def _workspace(self, n: int):
        import torch
        need = self.workspace_bytes(n)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    @staticmethod
    def _stream() -> int:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)

    def alloc_search(self, demand_mqps: Sequence[int], workers: int, slo_us: int, comm_us: int = 0, *,
                     flags: int = 0, begin: int = 0, end: Optional[int] = None) -> List[Result]:
        if end is None:
            end = self.num_candidates()
        m = len(demand_mqps)
        ws = self._workspace(m)
        out = (Result * m)()
        _check(lib().loki_alloc_search(self._h, _arr(C.c_int64, demand_mqps), m, workers, slo_us, comm_us, flags,
                                       begin, end, ws.data_ptr(), ws.numel(), self._stream(), out),
               "loki_alloc_search")
        return list(out)

    def alloc_search_static(self, demand_mqps: Sequence[int], workers: int, slo_us: int, comm_us: int = 0, *,
                            flags: int = 0, begin: int = 0, end: Optional[int] = None) -> List[Result]:
        """The search in the library's own static device scratch: no workspace, nothing allocated."""
        if end is None:
            end = self.num_candidates()
        m = len(demand_mqps)
        out = (Result * m)()
        _check(lib().loki_alloc_search_static(self._h, _arr(C.c_int64, demand_mqps), m, workers, slo_us, comm_us,
                                              flags, begin, end, self._stream(), out), "loki_alloc_search_static")
        return list(out)

    def alloc_search_enqueue(self, demand_mqps: Sequence[int], workers: int, slo_us: int, comm_us: int = 0, *,
                             flags: int = 0, begin: int = 0, end: Optional[int] = None, results=None):
        """Enqueue only; returns the torch uint8 tensor (32 bytes per demand point) the results land in."""
        import torch
        if end is None:
            end = self.num_candidates()
        m = len(demand_mqps)
        ws = self._workspace(m)
        if results is None:
            results = torch.empty(32 * m, dtype=torch.uint8, device="cuda")
        _check(lib().loki_alloc_search_enqueue(self._h, _arr(C.c_int64, demand_mqps), m, workers, slo_us, comm_us,
                                               flags, begin, end, ws.data_ptr(), ws.numel(), self._stream(),
                                               results.data_ptr()), "loki_alloc_search_enqueue")
        return results

    def alloc_eval(self, indices: Sequence[int], demand_mqps: int, workers: int, slo_us: int,
                   comm_us: int = 0) -> List[Eval]:
        n = len(indices)
        ws = self._workspace(n)
        out = (Eval * n)()
        _check(lib().loki_alloc_eval(self._h, _arr(C.c_uint64, indices), n, demand_mqps, workers, slo_us, comm_us,
                                     ws.data_ptr(), ws.numel(), self._stream(), out), "loki_alloc_eval")
        return list(out)

    def route_table(self, index: int, demand_mqps: int) -> Route:
        out = Route()
        _check(lib().loki_route_table(self._h, index, demand_mqps, C.byref(out)), "loki_route_table")
        return out

    def route_table_batch(self, indices: Sequence[int], demand_mqps: Sequence[int]) -> List[Route]:
        import torch
        n = len(indices)
        need = C.c_size_t()
        _check(lib().loki_route_workspace_bytes(self._h, n, C.byref(need)), "loki_route_workspace_bytes")
        ws = torch.empty(int(need.value), dtype=torch.uint8, device="cuda")
        out = (Route * n)()
        _check(lib().loki_route_table_batch(self._h, _arr(C.c_uint64, indices), _arr(C.c_int64, demand_mqps), n,
                                            ws.data_ptr(), ws.numel(), self._stream(), out), "loki_route_table_batch")
        return list(out)

    def plan_trace(self, trace_mqps: Sequence[int], alpha_ppm: int, workers: int, slo_us: int, comm_us: int = 0,
                   *, flags: int = 0) -> List[PlanStep]:
        n = len(trace_mqps)
        ws = self._workspace(n)
        out = (PlanStep * n)()
        _check(lib().loki_plan_trace(self._h, _arr(C.c_int64, trace_mqps), n, alpha_ppm, workers, slo_us, comm_us,
                                     flags, ws.data_ptr(), ws.numel(), self._stream(), out), "loki_plan_trace")
        return list(out)

    def last_search_ms(self) -> List[float]:
        """[per-task tables, main search kernel, final merge] of the last blocking search, in ms."""
        ms = (C.c_float * 3)()
        _check(lib().loki_last_search_ms(self._h, ms), "loki_last_search_ms")
        return [float(v) for v in ms]

    def last_search_fill_bits(self) -> int:
        """32 or 64: the integer width of the last per-lane search's fill."""
        b = C.c_int32()
        _check(lib().loki_last_search_fill_bits(self._h, C.byref(b)), "loki_last_search_fill_bits")
        return int(b.value)

    def last_search_plans_scored(self) -> int:
        """Plans whose score the kernels of the last search formed (see the header)."""
        n = C.c_uint64()
        _check(lib().loki_last_search_plans_scored(self._h, C.byref(n)), "loki_last_search_plans_scored")
        return int(n.value)


RATE_KINDS = {"v_mul_f64": 0, "v_add_f64": 1, "v_max_f64": 2, "search_mix": 3, "v_add_u32": 4, "v_fma_f64": 5,
              "v_rcp_f64": 6, "v_mul_lo_u32": 7, "v_mul_hi_u32": 8, "v_min_u32": 9, "ds_read_b64": 10}


PROBE_EXPORTS = ["loki_measure_valu_rate"]   # include/loki_probe.h, libloki_probe.so
_probe = None


def probe_lib():
    """The instruction-rate probe, a library of its own beside the search library."""
    global _probe
    if _probe is None:
        from . import build
        if not os.path.exists(build.PROBE_LIB):
            raise RuntimeError(f"{build.PROBE_LIB} is missing: run `python -m paper_2407_03583_amd.build` first")
        import torch  # noqa: F401  (its HIP runtime first, as for the search library)
        L = C.CDLL(build.PROBE_LIB)
        L.loki_measure_valu_rate.restype = C.c_int
        L.loki_measure_valu_rate.argtypes = [C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double),
                                             C.POINTER(C.c_int)]
        _probe = L
    return _probe


def measure_valu_rate(kind: str) -> float:
    """Sustained wavefront instructions per second of one vector-ALU instruction class."""
    import torch
    ws = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    rate, hip_error = C.c_double(), C.c_int(0)
    rc = probe_lib().loki_measure_valu_rate(RATE_KINDS[kind], ws.data_ptr(), ws.numel(),
                                            int(torch.cuda.current_stream().cuda_stream), C.byref(rate), C.byref(hip_error))
    if rc != 0:
        raise RuntimeError(f"loki_measure_valu_rate: error {rc} (HIP code {hip_error.value})")
    return float(rate.value)


def results_from_bytes(buf: bytes) -> List[Result]:
    n = len(buf) // C.sizeof(Result)
    return list((Result * n).from_buffer_copy(buf))
