"""ctypes access to the CPU checker (oracle/loki_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product's binding or kernels.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "loki_oracle.c")
_LIB = os.path.join(_HERE, "libloki_oracle.so")

MAX_TASKS = 8
MAX_VARIANTS = 8

BAD_WORKERS, BAD_DEMAND, BAD_EMPTY, BAD_LATENCY = 1, 2, 4, 8
UINT64_MAX = (1 << 64) - 1


def build(force: bool = False) -> str:
    """Compile the checker with gcc (no FMA contraction, OpenMP for the range split)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= max(os.path.getmtime(_SRC),
                                              os.path.getmtime(os.path.join(_HERE, "loki_oracle.h")))):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-Wextra", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class _Pipeline(C.Structure):
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


class EvalOut(C.Structure):
    _fields_ = [("infeasible", C.c_int32),
                ("workers", C.c_int32),
                ("accuracy", C.c_double),
                ("task_acc", C.c_double * MAX_TASKS),
                ("task_maxlat", C.c_int64 * MAX_TASKS),
                ("task_demand", C.c_int64 * MAX_TASKS),
                ("task_unserved", C.c_int64 * MAX_TASKS)]


class Best(C.Structure):
    _fields_ = [("index", C.c_uint64),
                ("accuracy", C.c_double),
                ("n_feasible", C.c_uint64),
                ("workers", C.c_int32),
                ("found", C.c_int32)]

    def as_tuple(self):
        return (int(self.index), float(self.accuracy), int(self.n_feasible), int(self.workers), int(self.found))


class Route(C.Structure):
    _fields_ = [("demand", C.c_int64 * MAX_TASKS),
                ("scale", C.c_int64 * MAX_TASKS),
                ("capacity", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("routed", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("leftover", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("unserved", C.c_int64 * MAX_TASKS),
                ("budget_us", (C.c_int64 * MAX_VARIANTS) * MAX_TASKS),
                ("prob", ((C.c_double * MAX_VARIANTS) * MAX_VARIANTS) * MAX_TASKS)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # A test may point at a deliberately broken build of the checker to show that the pins notice
        # (tests/test_oracle_mutants.py sets both variables for its subprocesses); LOKI_ORACLE_LIB alone
        # is ignored, so that no other process can end up with a checker that is not the in-tree one
        override = os.environ.get("LOKI_ORACLE_LIB") if os.environ.get("LOKI_ORACLE_MUTANT_TEST") == "1" else None
        if not override:
            build()
        L = C.CDLL(override or _LIB)
        P = C.POINTER(_Pipeline)
        L.lo_num_candidates.restype = C.c_uint64
        L.lo_num_candidates.argtypes = [P]
        L.lo_decode.restype = None
        L.lo_decode.argtypes = [P, C.c_uint64, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.lo_encode.restype = C.c_uint64
        L.lo_encode.argtypes = [P, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.lo_eval.restype = None
        L.lo_eval.argtypes = [P, C.c_uint64, C.c_int64, C.c_int32, C.c_int64, C.c_int64, C.POINTER(EvalOut)]
        L.lo_search.restype = None
        L.lo_search.argtypes = [P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, C.c_int, C.c_uint64,
                                C.c_uint64, C.c_uint64, C.c_int, C.POINTER(Best)]
        L.lo_search_tabulated.restype = None
        L.lo_search_tabulated.argtypes = [P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, C.c_int,
                                          C.c_uint64, C.c_uint64, C.c_int, C.POINTER(Best)]
        L.lo_route_table.restype = None
        L.lo_route_table.argtypes = [P, C.c_uint64, C.c_int64, C.POINTER(Route)]
        L.lo_max_threads.restype = C.c_int
        L.lo_max_threads.argtypes = []
        _lib = L
    return _lib


def _arr(ctype, values: Sequence[int]):
    return (ctype * max(1, len(values)))(*[int(v) for v in values])


class Problem:
    """Holds the C arrays of one pipeline (any object with the Table-1 input
    attributes: n_tasks, parent, fanout_q4, n_variants, n_batches, batch_size,
    max_replicas, acc_ppm, latency_us, thr_mqps)."""

    def __init__(self, pipeline):
        self.n_tasks = int(pipeline.n_tasks)
        self.n_variants = [int(v) for v in pipeline.n_variants]
        self._keep = {
            "parent": _arr(C.c_int32, pipeline.parent),
            "fanout_q4": _arr(C.c_int32, pipeline.fanout_q4),
            "n_variants": _arr(C.c_int32, pipeline.n_variants),
            "n_batches": _arr(C.c_int32, pipeline.n_batches),
            "batch_size": _arr(C.c_int32, pipeline.batch_size),
            "max_replicas": _arr(C.c_int32, pipeline.max_replicas),
            "acc_ppm": _arr(C.c_int32, pipeline.acc_ppm),
            "latency_us": _arr(C.c_int64, pipeline.latency_us),
            "thr_mqps": _arr(C.c_int64, pipeline.thr_mqps),
        }
        vf = getattr(pipeline, "variant_factor_q4", None)
        if vf is not None:
            self._keep["variant_factor_q4"] = _arr(C.c_int32, vf)
        pt = getattr(pipeline, "path_acc_ppm", None)
        if pt is not None:
            self._keep["path_acc_ppm"] = _arr(C.c_int32, pt)
        k = self._keep
        self.c = _Pipeline(self.n_tasks,
                           C.cast(k["parent"], C.POINTER(C.c_int32)),
                           C.cast(k["fanout_q4"], C.POINTER(C.c_int32)),
                           C.cast(k["n_variants"], C.POINTER(C.c_int32)),
                           C.cast(k["n_batches"], C.POINTER(C.c_int32)),
                           C.cast(k["batch_size"], C.POINTER(C.c_int32)),
                           C.cast(k["max_replicas"], C.POINTER(C.c_int32)),
                           C.cast(k["acc_ppm"], C.POINTER(C.c_int32)),
                           C.cast(k["latency_us"], C.POINTER(C.c_int64)),
                           C.cast(k["thr_mqps"], C.POINTER(C.c_int64)),
                           C.cast(k["variant_factor_q4"], C.POINTER(C.c_int32)) if vf is not None
                           else C.POINTER(C.c_int32)(),
                           1 if getattr(pipeline, "per_variant_batch", False) else 0,
                           C.cast(k["path_acc_ppm"], C.POINTER(C.c_int32)) if pt is not None
                           else C.POINTER(C.c_int32)(),
                           1 if getattr(pipeline, "latency_per_path", False) else 0)
        self.per_variant_batch = bool(getattr(pipeline, "per_variant_batch", False))

    def num_candidates(self) -> int:
        return int(lib().lo_num_candidates(C.byref(self.c)))

    def decode(self, index: int):
        x = (C.c_int32 * sum(self.n_variants))()
        b = (C.c_int32 * (sum(self.n_variants) if self.per_variant_batch else self.n_tasks))()
        lib().lo_decode(C.byref(self.c), index, x, b)
        return list(x), list(b)

    def encode(self, x: Sequence[int], batch_digit: Sequence[int]) -> int:
        return int(lib().lo_encode(C.byref(self.c), _arr(C.c_int32, x), _arr(C.c_int32, batch_digit)))

    def eval(self, index: int, demand_mqps: int, workers: int, slo_us: int, comm_us: int = 0) -> EvalOut:
        out = EvalOut()
        lib().lo_eval(C.byref(self.c), index, demand_mqps, workers, slo_us, comm_us, C.byref(out))
        return out

    def search(self, demand_mqps: int, workers: int, slo_us: int, comm_us: int = 0, *,
               tie_index_only: bool = False, begin: int = 0, end: int | None = None,
               stride: int = 1, threads: int | None = None) -> Best:
        if end is None:
            end = self.num_candidates()
        if threads is None:
            threads = max_threads()
        out = Best()
        lib().lo_search(C.byref(self.c), demand_mqps, workers, slo_us, comm_us, int(tie_index_only),
                        begin, end, stride, threads, C.byref(out))
        return out

    def search_tabulated(self, demand_mqps: int, workers: int, slo_us: int, comm_us: int = 0, *,
                         tie_index_only: bool = False, begin: int = 0, end: int | None = None,
                         threads: int | None = None) -> Best:
        if end is None:
            end = self.num_candidates()
        if threads is None:
            threads = max_threads()
        out = Best()
        lib().lo_search_tabulated(C.byref(self.c), demand_mqps, workers, slo_us, comm_us,
                                  int(tie_index_only), begin, end, threads, C.byref(out))
        return out

    def route_table(self, index: int, demand_mqps: int) -> Route:
        out = Route()
        lib().lo_route_table(C.byref(self.c), index, demand_mqps, C.byref(out))
        return out


def max_threads() -> int:
    return int(lib().lo_max_threads())
