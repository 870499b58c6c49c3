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
    first);
  * scaling up on arrival (Section 3.3.2: add an Aggregator, assign the entire
    job again, repeat until the job no longer loses speed): the job was placed
    where the estimates said it would not lose speed and lost speed all the
    same, so running the same estimates again over one more (empty) Aggregator
    would put every task back where it was -- best fit never prefers the
    emptiest destination.  The reading taken: the Aggregators added for this
    job by scale-up steps are offered FIRST, oldest first, each to every task
    it still qualifies for (loss test, F >= e_t); only a task that none of them
    holds goes through Pseudocode 1 over the other Aggregators.  Every step
    then takes up to one cycle's worth of the job's aggregations off the
    shared Aggregators, and the loop ends at the latest when the job sits on
    Aggregators of its own, which is its standalone placement.
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
        self.own: Dict[int, List[int]] = {}   # job -> Aggregators added for it by scale-up, oldest first
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

    def _release(self, n: int) -> None:
        """Hand an (empty) Aggregator back; no job keeps it as one of its own."""
        del self.aggs[n]
        for k in list(self.own):
            self.own[k] = [m for m in self.own[k] if m != n]
            if not self.own[k]:
                del self.own[k]

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
        self.own.pop(k, None)
        for n in sorted(self.aggs):
            if self.aggs[n].empty():
                self._release(n)
                released.append(n)
        while len(self.aggs) > 1:
            victim = min(self.aggs, key=lambda n: (self.busy(n) / self.cycle(n), -n))
            moved = self._drain(victim)
            if not moved:
                break
            self._release(victim)
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
    def scale_up_job(self, k: int) -> Tuple[int, int]:
        """The monitored job k runs slower than standalone: allocate one more
        Aggregator for it and assign the whole job again, task by task in task-id
        order.  The Aggregators added for k (by earlier calls and by this one) are
        offered first, oldest first: a task goes to the first of them that passes
        the loss test and has F >= e_t; a task that none of them holds goes through
        Pseudocode 1 over the other Aggregators.  Aggregators left empty are
        released.  Returns (the new Aggregator's id, the number of k's tasks whose
        Aggregator changed); the caller repeats while the measured loss stays above
        LossLimit and the second number is not zero."""
        mine = sorted((t, e) for t, (n, j, e) in self.where.items() if j == k)
        before = {t: self.where[t][0] for t, _ in mine}
        for t, e in mine:
            n = self.where[t][0]
            self.aggs[n].tasks[k].remove((t, e))
            if not self.aggs[n].tasks[k]:
                del self.aggs[n].tasks[k]
        fresh = self.allocate()
        self.own.setdefault(k, []).append(fresh)
        for t, e in mine:
            n = None
            for cand in self.own[k]:
                est = self.estimate(cand, k)
                if est is not None and est[1] >= e:
                    n = cand
                    break
            if n is None:
                n = self.choose(k, e, exclude=tuple(self.own[k]))
            self._place(n, k, e, task=t)
        for n in sorted(self.aggs):
            if self.aggs[n].empty():
                self._release(n)
        moved = sum(1 for t, _ in mine if self.where[t][0] != before[t])
        return fresh, moved

    # -- two-level placement (Section 3.3.3) ------------------------------------
    @staticmethod
    def best_fit_cluster(free: List[float], demand: float) -> Optional[int]:
        """The cluster with sufficient but the least free resource; None if none fits."""
        ok = [(f, i) for i, f in enumerate(free) if f >= demand]
        return min(ok)[1] if ok else None


class PMasterOracle:
    """Aggregator clusters (Section 3.3.3).  The pool of Aggregators is split
    into independent clusters; each has a controller that runs the assignment
    scheme over its own Aggregators only (one SchedulerOracle per cluster, with
    Aggregator and task ids local to the cluster).  pMaster keeps, on its own
    side, the remaining free resource of every cluster and places a new job in
    two steps: it forwards the job to the best-fit cluster by the job's total
    demand, then that cluster's controller assigns the job's model aggregations;
    a job takes resource from one cluster only.  When a job exits, its
    controller reports it and pMaster gives the job's demand back to the cluster.

    Readings where the text is silent:
      * unit of "CPU resource": Aggregators.  A cluster of capacity M offers M
        units; a job with profiled duration D and tasks e_t consumes
        sum(e_t) / D of one Aggregator (its aggregation time per unit of time);
        free = capacity - sum of the demands of the jobs forwarded there.  This
        is pMaster's own book, kept from profiled job information: it does not
        look at how the controller packed the tasks;
      * ties between equally free clusters go to the lowest cluster id;
      * if no cluster has room the job is not placed (None): adding clusters or
        Aggregators to a cluster is the periodic scaling policy, not part of
        this step;
      * scaling a job up happens inside its cluster and leaves its demand, and
        therefore pMaster's book, unchanged.
    """

    def __init__(self, loss_limit: float = LOSS_LIMIT_DEFAULT):
        self.loss_limit = loss_limit
        self.capacity: List[float] = []
        self.controllers: List[SchedulerOracle] = []
        self.jobs: Dict[int, Tuple[int, int, float]] = {}   # job -> (cluster, controller's job id, demand)
        self.next_job = 0

    def add_cluster(self, capacity: float) -> int:
        assert capacity > 0
        self.capacity.append(capacity)
        self.controllers.append(SchedulerOracle(self.loss_limit))
        return len(self.capacity) - 1

    def used(self, c: int) -> float:
        total = 0.0
        for j in sorted(self.jobs):
            if self.jobs[j][0] == c:
                total += self.jobs[j][2]
        return total

    def free(self, c: int) -> float:
        return self.capacity[c] - self.used(c)

    @staticmethod
    def demand(D: float, es: List[float]) -> float:
        total = 0.0
        for e in es:
            total += e
        return total / D

    def forward_job(self, D: float, es: List[float]) -> Optional[Tuple[int, int, List[Tuple[int, int]]]]:
        """A new job with profiled iteration D and task execution times es.
        -> (job id, cluster, [(task id, Aggregator)] in the cluster's own ids), or
        None if no cluster has room for its demand."""
        need = self.demand(D, es)
        c = SchedulerOracle.best_fit_cluster([self.free(i) for i in range(len(self.capacity))], need)
        if c is None:
            return None
        ctl = self.controllers[c]
        local = ctl.add_job(D)
        placed = [ctl.assign(local, e) for e in es]
        j = self.next_job
        self.next_job += 1
        self.jobs[j] = (c, local, need)
        return j, c, placed

    def job_exit(self, j: int) -> Tuple[int, List[int]]:
        """The controller removes the job (releasing and recycling Aggregators
        inside its cluster) and reports the exit; pMaster forgets the job, which
        gives its demand back.  -> (cluster, Aggregators released there)."""
        c, local, _ = self.jobs.pop(j)
        return c, self.controllers[c].remove_job(local)

    def scale_up_job(self, j: int) -> Tuple[int, int]:
        c, local, _ = self.jobs[j]
        return self.controllers[c].scale_up_job(local)
