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
    "ps_pmaster_create", "ps_pmaster_destroy", "ps_pmaster_add_cluster", "ps_pmaster_n_clusters",
    "ps_pmaster_forward_job", "ps_pmaster_job_exit", "ps_pmaster_scale_up_job", "ps_pmaster_cluster_info",
    "ps_pmaster_job_info", "ps_pmaster_controller",
]


class ClusterStats(C.Structure):
    _fields_ = [("capacity", C.c_double), ("used", C.c_double), ("free_resource", C.c_double),
                ("n_jobs", C.c_int32), ("n_aggregators", C.c_int32)]


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
        L.ps_sched_scale_up_job.argtypes = [vp, i32, P(i32), P(i32)]
        L.ps_sched_aggregator_info.argtypes = [vp, i32, P(AggStats)]
        L.ps_sched_job_info.argtypes = [vp, i32, P(JobStats)]
        L.ps_sched_task_info.argtypes = [vp, i32, P(i32), P(i32), P(dbl)]
        L.ps_sched_aggregators.argtypes = [vp, P(i32), i32, P(i32)]
        L.ps_sched_cycle_plan.argtypes = [vp, i32, P(Wave), i32, P(i32), P(i32), i32, P(i32)]
        L.ps_sched_admit_late.argtypes = [dbl, dbl, dbl, dbl]
        L.ps_sched_best_fit_cluster.argtypes = [P(dbl), i32, dbl]
        L.ps_pmaster_create.argtypes = [dbl, P(vp)]
        L.ps_pmaster_destroy.argtypes = [vp]
        L.ps_pmaster_destroy.restype = None
        L.ps_pmaster_add_cluster.argtypes = [vp, dbl, P(i32)]
        L.ps_pmaster_n_clusters.argtypes = [vp]
        L.ps_pmaster_forward_job.argtypes = [vp, dbl, P(dbl), i32, P(i32), P(i32), P(i32), P(i32)]
        L.ps_pmaster_job_exit.argtypes = [vp, i32, P(i32), P(i32), i32, P(i32)]
        L.ps_pmaster_scale_up_job.argtypes = [vp, i32, P(i32), P(i32)]
        L.ps_pmaster_cluster_info.argtypes = [vp, i32, P(ClusterStats)]
        L.ps_pmaster_job_info.argtypes = [vp, i32, P(i32), P(i32), P(dbl)]
        L.ps_pmaster_controller.argtypes = [vp, i32]
        for n in SCHED_EXPORTS:
            if n not in ("ps_sched_destroy", "ps_pmaster_destroy", "ps_pmaster_controller"):
                getattr(L, n).restype = i32
        L.ps_pmaster_controller.restype = vp
        _ready = True
    return L


class Scheduler:
    def __init__(self, loss_limit: float = 0.0, _borrowed: Optional[int] = None):
        self.L = _lib()
        self.owned = _borrowed is None
        if self.owned:
            self.h = C.c_void_p()
            self._check(self.L.ps_sched_create(loss_limit, C.byref(self.h)))
        else:
            self.h = C.c_void_p(_borrowed)     # a cluster's controller: pMaster owns it

    def _check(self, st: int) -> int:
        if st < 0:
            raise PsError(st, self.L.ps_strerror(st).decode())
        return st

    def close(self) -> None:
        if self.h and self.owned:
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

    def scale_up_job(self, job: int) -> Tuple[int, int]:
        """-> (the new Aggregator, how many of the job's tasks changed Aggregator)."""
        n, moved = C.c_int32(), C.c_int32()
        self._check(self.L.ps_sched_scale_up_job(self.h, job, C.byref(n), C.byref(moved)))
        return n.value, moved.value

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


class PMaster:
    """ps_pmaster_*: Aggregator clusters, one Scheduler (controller) per cluster."""

    def __init__(self, loss_limit: float = 0.0):
        self.L = _lib()
        self.h = C.c_void_p()
        self._check(self.L.ps_pmaster_create(loss_limit, C.byref(self.h)))

    def _check(self, st: int) -> int:
        if st < 0:
            raise PsError(st, self.L.ps_strerror(st).decode())
        return st

    def close(self) -> None:
        if self.h:
            self.L.ps_pmaster_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_cluster(self, capacity: float) -> int:
        c = C.c_int32()
        self._check(self.L.ps_pmaster_add_cluster(self.h, capacity, C.byref(c)))
        return c.value

    def n_clusters(self) -> int:
        return self._check(self.L.ps_pmaster_n_clusters(self.h))

    def forward_job(self, D: float, es: List[float]) -> Optional[Tuple[int, int, List[Tuple[int, int]]]]:
        """-> (job, cluster, [(task, Aggregator)] in the cluster's ids); None if no cluster has room."""
        n = len(es)
        arr = (C.c_double * max(n, 1))(*es)
        job, cl = C.c_int32(), C.c_int32()
        tasks, aggs = (C.c_int32 * max(n, 1))(), (C.c_int32 * max(n, 1))()
        st = self.L.ps_pmaster_forward_job(self.h, D, arr, n, C.byref(job), C.byref(cl), tasks, aggs)
        if st == -15:
            return None
        self._check(st)
        return job.value, cl.value, list(zip(tasks[:n], aggs[:n]))

    def job_exit(self, job: int) -> Tuple[int, List[int]]:
        cl, n = C.c_int32(), C.c_int32()
        cap = 1024
        out = (C.c_int32 * cap)()
        self._check(self.L.ps_pmaster_job_exit(self.h, job, C.byref(cl), out, cap, C.byref(n)))
        return cl.value, list(out[:n.value])

    def scale_up_job(self, job: int) -> Tuple[int, int]:
        n, moved = C.c_int32(), C.c_int32()
        self._check(self.L.ps_pmaster_scale_up_job(self.h, job, C.byref(n), C.byref(moved)))
        return n.value, moved.value

    def cluster_info(self, cluster: int) -> ClusterStats:
        out = ClusterStats()
        self._check(self.L.ps_pmaster_cluster_info(self.h, cluster, C.byref(out)))
        return out

    def job_info(self, job: int) -> Tuple[int, int, float]:
        cl, local, d = C.c_int32(), C.c_int32(), C.c_double()
        self._check(self.L.ps_pmaster_job_info(self.h, job, C.byref(cl), C.byref(local), C.byref(d)))
        return cl.value, local.value, d.value

    def controller(self, cluster: int) -> Scheduler:
        """The cluster's controller for inspection (borrowed: valid while this object lives)."""
        h = self.L.ps_pmaster_controller(self.h, cluster)
        if not h:
            raise PsError(-3, "no such cluster")
        return Scheduler(_borrowed=h)
