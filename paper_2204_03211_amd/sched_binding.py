"""ctypes binding of the scheduling entry points (include/ps_sched.h): one method
per C function, argument marshalling only."""
from __future__ import annotations

import ctypes as C
from fractions import Fraction
from typing import List, Optional, Tuple

from .binding import PsError, load_library


class AggStats(C.Structure):
    _fields_ = [("cycle", C.c_double), ("busy", C.c_double), ("free_time", C.c_double),
                ("n_jobs", C.c_int32), ("n_tasks", C.c_int32)]


class JobStats(C.Structure):
    _fields_ = [("D", C.c_double), ("d", C.c_double), ("loss", C.c_double),
                ("n_tasks", C.c_int32), ("n_aggregators", C.c_int32)]


class Wave(C.Structure):
    _fields_ = [("num", C.c_int64), ("den", C.c_int64), ("first", C.c_int32), ("count", C.c_int32)]


SCHED_EXPORTS = [
    "ps_sched_create", "ps_sched_destroy", "ps_sched_add_job", "ps_sched_assign", "ps_sched_estimate",
    "ps_sched_remove_job", "ps_sched_scale_up_job", "ps_sched_aggregator_info", "ps_sched_job_info", "ps_sched_task_info",
    "ps_sched_aggregators", "ps_sched_cycle_plan", "ps_sched_admit_late", "ps_sched_best_fit_cluster",
]

_ready = False


def _lib():
    global _ready
    L = load_library()
    if not _ready:
        vp, i32, dbl, P = C.c_void_p, C.c_int32, C.c_double, C.POINTER
        L.ps_sched_create.argtypes = [dbl, P(vp)]
        L.ps_sched_destroy.argtypes = [vp]
        L.ps_sched_destroy.restype = None
        L.ps_sched_add_job.argtypes = [vp, dbl, P(i32)]
        L.ps_sched_assign.argtypes = [vp, i32, dbl, P(i32), P(i32)]
        L.ps_sched_estimate.argtypes = [vp, i32, i32, P(dbl), P(dbl)]
        L.ps_sched_remove_job.argtypes = [vp, i32, P(i32), i32, P(i32)]
        L.ps_sched_scale_up_job.argtypes = [vp, i32, P(i32)]
        L.ps_sched_aggregator_info.argtypes = [vp, i32, P(AggStats)]
        L.ps_sched_job_info.argtypes = [vp, i32, P(JobStats)]
        L.ps_sched_task_info.argtypes = [vp, i32, P(i32), P(i32), P(dbl)]
        L.ps_sched_aggregators.argtypes = [vp, P(i32), i32, P(i32)]
        L.ps_sched_cycle_plan.argtypes = [vp, i32, P(Wave), i32, P(i32), P(i32), i32, P(i32)]
        L.ps_sched_admit_late.argtypes = [dbl, dbl, dbl, dbl]
        L.ps_sched_best_fit_cluster.argtypes = [P(dbl), i32, dbl]
        for n in SCHED_EXPORTS:
            if n != "ps_sched_destroy":
                getattr(L, n).restype = i32
        _ready = True
    return L


class Scheduler:
    def __init__(self, loss_limit: float = 0.0):
        self.L = _lib()
        self.h = C.c_void_p()
        self._check(self.L.ps_sched_create(loss_limit, C.byref(self.h)))

    def _check(self, st: int) -> int:
        if st < 0:
            raise PsError(st, self.L.ps_strerror(st).decode())
        return st

    def close(self) -> None:
        if self.h:
            self.L.ps_sched_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_job(self, D: float) -> int:
        j = C.c_int32()
        self._check(self.L.ps_sched_add_job(self.h, D, C.byref(j)))
        return j.value

    def assign(self, job: int, e: float) -> Tuple[int, int]:
        t, n = C.c_int32(), C.c_int32()
        self._check(self.L.ps_sched_assign(self.h, job, e, C.byref(t), C.byref(n)))
        return t.value, n.value

    def estimate(self, aggregator: int, job: int) -> Optional[Tuple[float, float]]:
        c, f = C.c_double(), C.c_double()
        ok = self._check(self.L.ps_sched_estimate(self.h, aggregator, job, C.byref(c), C.byref(f)))
        return (c.value, f.value) if ok else None

    def remove_job(self, job: int) -> List[int]:
        n = C.c_int32()
        cap = 1024
        out = (C.c_int32 * cap)()
        self._check(self.L.ps_sched_remove_job(self.h, job, out, cap, C.byref(n)))
        return list(out[:n.value])

    def scale_up_job(self, job: int) -> int:
        n = C.c_int32()
        self._check(self.L.ps_sched_scale_up_job(self.h, job, C.byref(n)))
        return n.value

    def aggregator_info(self, aggregator: int) -> AggStats:
        out = AggStats()
        self._check(self.L.ps_sched_aggregator_info(self.h, aggregator, C.byref(out)))
        return out

    def job_info(self, job: int) -> JobStats:
        out = JobStats()
        self._check(self.L.ps_sched_job_info(self.h, job, C.byref(out)))
        return out

    def task_info(self, task: int) -> Tuple[int, int, float]:
        a, j, e = C.c_int32(), C.c_int32(), C.c_double()
        self._check(self.L.ps_sched_task_info(self.h, task, C.byref(a), C.byref(j), C.byref(e)))
        return a.value, j.value, e.value

    def aggregators(self) -> List[int]:
        n = C.c_int32()
        st = self.L.ps_sched_aggregators(self.h, None, 0, C.byref(n))
        if st not in (0, -12):
            self._check(st)
        out = (C.c_int32 * max(n.value, 1))()
        self._check(self.L.ps_sched_aggregators(self.h, out, n.value, C.byref(n)))
        return list(out[:n.value])

    def cycle_plan(self, aggregator: int) -> List[Tuple[Fraction, List[int]]]:
        nw, nj = C.c_int32(), C.c_int32()
        st = self.L.ps_sched_cycle_plan(self.h, aggregator, None, 0, C.byref(nw), None, 0, C.byref(nj))
        if st not in (0, -12):
            self._check(st)
        waves = (Wave * max(nw.value, 1))()
        jobs = (C.c_int32 * max(nj.value, 1))()
        self._check(self.L.ps_sched_cycle_plan(self.h, aggregator, waves, nw.value, C.byref(nw),
                                               jobs, nj.value, C.byref(nj)))
        return [(Fraction(w.num, w.den), list(jobs[w.first:w.first + w.count])) for w in waves[:nw.value]]

    @staticmethod
    def admit_late(cycle: float, elapsed: float, remaining_scheduled: float, e_late: float) -> bool:
        return bool(_lib().ps_sched_admit_late(cycle, elapsed, remaining_scheduled, e_late))

    @staticmethod
    def best_fit_cluster(free_time: List[float], demand: float) -> Optional[int]:
        arr = (C.c_double * max(len(free_time), 1))(*free_time)
        i = _lib().ps_sched_best_fit_cluster(arr, len(free_time), demand)
        return None if i < 0 else i
