"""Oracle for the assignment and scaling of model aggregations -- TEST
INFRASTRUCTURE ONLY (see oracle/__init__.py for who may import this).

A plain statement, in the paper's notation, of Section 3.3 ("Model Aggregation
Management"): cyclic execution, the assignment heuristic of Pseudocode 1, the
handling of late requests, and Aggregator scaling on job arrival and exit.
Slow and obvious on purpose: sets and dictionaries, everything recomputed from
scratch at every step.

Notation (Table "Notations in the assignment scheme"):
    D_j   profiled (standalone) iteration duration of job j
    C_n   execution cycle of Aggregator n = the largest D_j among its jobs
    d_j   iteration duration of job j when it runs floor(C/D_j) times per cycle
    e_t   execution time of task t (one model aggregation per iteration)
    F_n   free time of Aggregator n within one cycle

Readings where the printed pseudocode is garbled or silent:
  * the loss test applies to every job already on the Aggregator AND to the
    new task's job k (the printed test sits outside the loop over jobs);
  * C^new in the free-slot formula is C^est;
  * the set operations printed as intersections are unions;
  * "best fit" is the Aggregator with the least estimated free time that still
    holds e_t (the text's wording); ties go to the lowest Aggregator id;
  * F^est counts the tasks already assigned, and e_t is compared against it;
  * loss is compared with >= LossLimit, as printed;
  * "least-loaded" Aggregator on recycling = smallest busy time per cycle
    divided by the cycle (ties to the highest id, so that younger Aggregators go
    first).
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Dict, List, Optional, Tuple

LOSS_LIMIT_DEFAULT = 0.1  # Section 3.3.1: "LossLimit, default is 0.1"


def iteration_duration(C: float, D: float) -> float:
    """d_j of a job with profiled duration D on an Aggregator of cycle C: the job
    runs floor(C/D) times per cycle, evenly spaced."""
    return max(D, C / math.floor(C / D))


def loss(d: float, D: float) -> float:
    return (d - D) / d


class Aggregator:
    def __init__(self, ident: int):
        self.id = ident
        self.tasks: Dict[int, List[Tuple[int, float]]] = {}  # job -> [(task id, e_t)]

    def jobs(self) -> List[int]:
        return sorted(self.tasks)

    def empty(self) -> bool:
        return not self.tasks


class SchedulerOracle:
    def __init__(self, loss_limit: float = LOSS_LIMIT_DEFAULT):
        self.loss_limit = loss_limit
        self.D: Dict[int, float] = {}
        self.aggs: Dict[int, Aggregator] = {}
        self.where: Dict[int, Tuple[int, int, float]] = {}   # task id -> (aggregator, job, e_t)
        self.next_agg = 0
        self.next_task = 0
        self.next_job = 0

    # -- bookkeeping ----------------------------------------------------------
    def add_job(self, D: float) -> int:
        assert D > 0
        j = self.next_job
        self.next_job += 1
        self.D[j] = D
        return j

    def cycle(self, n: int) -> float:
        a = self.aggs[n]
        return max((self.D[j] for j in a.tasks), default=0.0)

    def busy(self, n: int, C: Optional[float] = None) -> float:
        """W_n: time spent aggregating within one cycle of length C."""
        a = self.aggs[n]
        C = self.cycle(n) if C is None else C
        total = 0.0
        for j in a.jobs():
            d = iteration_duration(C, self.D[j])
            total += math.floor(C / d) * sum(e for _, e in a.tasks[j])
        return total

    def free(self, n: int) -> float:
        return self.cycle(n) - self.busy(n)

    def job_duration(self, j: int) -> float:
        """d_j over all Aggregators holding tasks of j (the slowest one counts)."""
        ds = [iteration_duration(self.cycle(n), self.D[j]) for n, a in self.aggs.items() if j in a.tasks]
        return max(ds, default=self.D[j])

    def job_loss(self, j: int) -> float:
        return loss(self.job_duration(j), self.D[j])

    # -- Pseudocode 1 ---------------------------------------------------------
    def estimate(self, n: int, k: int) -> Optional[Tuple[float, float]]:
        """(C_est, F_est) of Aggregator n if a task of job k were added, or None
        if some job there (or k) would lose LossLimit or more of its speed."""
        a = self.aggs[n]
        C_est = max(self.cycle(n), self.D[k])
        for j in set(a.tasks) | {k}:
            d = iteration_duration(C_est, self.D[j])
            if loss(d, self.D[j]) >= self.loss_limit:
                return None
        return C_est, C_est - self.busy(n, C_est)

    def allocate(self) -> int:
        n = self.next_agg
        self.next_agg += 1
        self.aggs[n] = Aggregator(n)
        return n

    def _place(self, n: int, k: int, e: float, task: Optional[int] = None) -> int:
        if task is None:
            task = self.next_task
            self.next_task += 1
        self.aggs[n].tasks.setdefault(k, []).append((task, e))
        self.where[task] = (n, k, e)
        return task

    def choose(self, k: int, e: float, allow_new: bool = True, exclude: Tuple[int, ...] = ()
               ) -> Optional[int]:
        """The Aggregator Pseudocode 1 picks for a task (e) of job k; allocates
        one if none qualifies and allow_new; None if none and not allow_new."""
        fits: List[Tuple[float, int]] = []
        for n in sorted(self.aggs):
            if n in exclude:
                continue
            est = self.estimate(n, k)
            if est is None:
                continue
            _, F = est
            if F >= e:
                fits.append((F, n))
        if fits:
            return min(fits)[1]
        return self.allocate() if allow_new else None

    def assign(self, k: int, e: float) -> Tuple[int, int]:
        """Assign a new task of job k with execution time e.  -> (task id, aggregator)."""
        n = self.choose(k, e)
        return self._place(n, k, e), n

    # -- cyclic execution -------------------------------------------------------
    def cycle_plan(self, n: int) -> List[Tuple[Fraction, List[int]]]:
        """The waves of one cycle of Aggregator n: [(start as a fraction of the
        cycle, jobs whose aggregations run in that wave)].  A job with
        floor(C/D_j) = r runs at fractions 0, 1/r, ..., (r-1)/r."""
        C = self.cycle(n)
        at: Dict[Fraction, List[int]] = {}
        for j in self.aggs[n].jobs():
            r = math.floor(C / self.D[j])
            for i in range(r):
                at.setdefault(Fraction(i, r), []).append(j)
        return [(f, sorted(js)) for f, js in sorted(at.items())]

    # -- late requests (Section 3.3.1, "Handling Outliers") ---------------------
    @staticmethod
    def admit_late(C: float, elapsed: float, remaining_scheduled: float, e_late: float) -> bool:
        """A request that missed its slot runs in the current cycle only if, after
        reserving time for the requests still scheduled in this cycle, enough of
        the cycle is left for it; otherwise it waits for the next cycle."""
        return (C - elapsed) - remaining_scheduled >= e_late

    # -- scaling on job exit (Section 3.3.2) ------------------------------------
    def remove_job(self, k: int) -> List[int]:
        """Job exit: drop its tasks, release empty Aggregators, then try to drain
        the least-loaded Aggregators one at a time into the others without
        allocating.  Returns the ids of the Aggregators released."""
        released: List[int] = []
        for n in sorted(self.aggs):
            a = self.aggs[n]
            for t, _ in a.tasks.pop(k, []):
                del self.where[t]
        del self.D[k]
        for n in sorted(self.aggs):
            if self.aggs[n].empty():
                del self.aggs[n]
                released.append(n)
        while len(self.aggs) > 1:
            victim = min(self.aggs, key=lambda n: (self.busy(n) / self.cycle(n), -n))
            moved = self._drain(victim)
            if not moved:
                break
            del self.aggs[victim]
            released.append(victim)
        return released

    def _drain(self, victim: int) -> bool:
        """Move every task of victim elsewhere (largest first); undo on failure."""
        a = self.aggs[victim]
        todo = sorted(((e, t, j) for j, ts in a.tasks.items() for t, e in ts), key=lambda x: (-x[0], x[1]))
        done: List[Tuple[int, int, int, float]] = []
        for e, t, j in todo:
            n = self.choose(j, e, allow_new=False, exclude=(victim,))
            if n is None:
                for t2, n2, j2, e2 in done:           # roll back
                    self.aggs[n2].tasks[j2].remove((t2, e2))
                    if not self.aggs[n2].tasks[j2]:
                        del self.aggs[n2].tasks[j2]
                    self.where[t2] = (victim, j2, e2)
                return False
            self._place(n, j, e, task=t)
            done.append((t, n, j, e))
        a.tasks.clear()
        return True

    # -- scaling on job arrival (Section 3.3.2) ---------------------------------
    def scale_up_job(self, k: int) -> int:
        """The monitored job k runs slower than standalone: allocate one more
        Aggregator and assign the whole job again, task by task in task-id order,
        with the new (empty) Aggregator among the destinations.  The caller
        repeats this while the measured loss stays above LossLimit.  Returns the
        new Aggregator's id; Aggregators that end up empty are released."""
        mine = sorted((t, e) for t, (n, j, e) in self.where.items() if j == k)
        for t, e in mine:
            n = self.where[t][0]
            self.aggs[n].tasks[k].remove((t, e))
            if not self.aggs[n].tasks[k]:
                del self.aggs[n].tasks[k]
        fresh = self.allocate()
        for t, e in mine:
            n = self.choose(k, e)
            self._place(n, k, e, task=t)
        for n in sorted(self.aggs):
            if self.aggs[n].empty():
                del self.aggs[n]
        return fresh

    # -- two-level placement (Section 3.3.3) ------------------------------------
    @staticmethod
    def best_fit_cluster(free: List[float], demand: float) -> Optional[int]:
        """The cluster with sufficient but the least free time; None if none fits."""
        ok = [(f, i) for i, f in enumerate(free) if f >= demand]
        return min(ok)[1] if ok else None
