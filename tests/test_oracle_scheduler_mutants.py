"""The scheduling pins must bite: plant one plausible mistake at a time in a
copy of the scheduling oracle's source (in memory, on the CPU), run the pins of
test_oracle_scheduler against the mutated copy, and check that at least one
fails.  The unmutated copy must pass them all."""
import os
import signal
import types

import pytest

import oracle.scheduler as good
import test_oracle_scheduler as T

SRC = open(os.path.join(os.path.dirname(good.__file__), "scheduler.py")).read()

MUTANTS = {
    "cycle is the shortest iteration": (
        "return max((self.D[j] for j in a.tasks), default=0.0)",
        "return min((self.D[j] for j in a.tasks), default=0.0)"),
    "runs per cycle rounded up": (
        "return max(D, C / math.floor(C / D))", "return max(D, C / math.ceil(C / D))"),
    "loss relative to the standalone duration": ("return (d - D) / d", "return (d - D) / D"),
    "loss limit exclusive": (
        "if loss(d, self.D[j]) >= self.loss_limit:", "if loss(d, self.D[j]) > self.loss_limit:"),
    "arriving job's own loss ignored": ("for j in set(a.tasks) | {k}:", "for j in set(a.tasks):"),
    "only the arriving job's loss checked": ("for j in set(a.tasks) | {k}:", "for j in {k}:"),
    "estimated cycle ignores the arriving job": (
        "C_est = max(self.cycle(n), self.D[k])", "C_est = max(self.cycle(n), 0.0) or self.D[k]"),
    "busy time counts each task once": (
        "total += math.floor(C / d) * sum(e for _, e in a.tasks[j])",
        "total += sum(e for _, e in a.tasks[j])"),
    "free time counts the new task already": (
        "return C_est, C_est - self.busy(n, C_est)", "return C_est, C_est - self.busy(n, C_est) - 0.5"),
    "worst fit": ("return min(fits)[1]", "return max(fits)[1]"),
    "first fit": ("return min(fits)[1]", "return fits[0][1]"),
    "ties to the highest id": ("fits.append((F, n))", "fits.append((F, -n))\n        fits = [(f, abs(m)) for f, m in fits] if False else fits"),
    "fit needs strictly more room": ("if F >= e:", "if F > e:"),
    "never allocates": (
        "return self.allocate() if allow_new else None", "return None"),
    "plan runs every job once": ("r = math.floor(C / self.D[j])\n", "r = 1\n"),
    "plan spacing off by one": ("at.setdefault(Fraction(i, r), [])", "at.setdefault(Fraction(i, r + 1), [])"),
    "late request ignores scheduled work": (
        "return (C - elapsed) - remaining_scheduled >= e_late", "return (C - elapsed) >= e_late"),
    "late request ignores elapsed time": (
        "return (C - elapsed) - remaining_scheduled >= e_late", "return C - remaining_scheduled >= e_late"),
    "exit does not recycle": ("        while len(self.aggs) > 1:\n", "        while False:\n"),
    "exit keeps empty Aggregators": (
        "            if self.aggs[n].empty():\n                self._release(n)\n                released.append(n)\n        while",
        "            pass\n        while"),
    "drains the most loaded": (
        "victim = min(self.aggs, key=lambda n: (self.busy(n) / self.cycle(n), -n))",
        "victim = max(self.aggs, key=lambda n: (self.busy(n) / self.cycle(n), -n))"),
    "drain ties to the lowest id": (
        "key=lambda n: (self.busy(n) / self.cycle(n), -n))", "key=lambda n: (self.busy(n) / self.cycle(n), n))"),
    "drain may allocate": (
        "n = self.choose(j, e, allow_new=False, exclude=(victim,))",
        "n = self.choose(j, e, allow_new=True, exclude=(victim,))"),
    "drain may pick the victim": (
        "n = self.choose(j, e, allow_new=False, exclude=(victim,))", "n = self.choose(j, e, allow_new=False)"),
    "failed drain not rolled back": ("                for t2, n2, j2, e2 in done:           # roll back\n",
                                     "                for t2, n2, j2, e2 in []:\n"),
    "scale-up adds nothing": ("        fresh = self.allocate()\n", "        fresh = max(self.aggs)\n"),
    "scale-up runs plain best fit again": ("            for cand in self.own[k]:\n", "            for cand in []:\n"),
    "scale-up offers the newest Aggregator first": (
        "            for cand in self.own[k]:\n", "            for cand in reversed(self.own[k]):\n"),
    "own Aggregators skip the room test": (
        "if est is not None and est[1] >= e:", "if est is not None:"),
    "own Aggregators skip the loss test": (
        "                est = self.estimate(cand, k)\n",
        "                C_ = max(self.cycle(cand), self.D[k])\n                est = (C_, C_ - self.busy(cand, C_))\n"),
    "scale-up reports every task as moved": (
        "moved = sum(1 for t, _ in mine if self.where[t][0] != before[t])", "moved = len(mine)"),
    "released Aggregators stay on a job's own list": (
        "self.own[k] = [m for m in self.own[k] if m != n]", "self.own[k] = list(self.own[k])"),
    "exit not reported to pMaster": ("c, local, _ = self.jobs.pop(j)", "c, local, _ = self.jobs[j]"),
    "demand is the plain sum of execution times": ("        return total / D\n", "        return total\n"),
    "job registered before the cluster is found": (
        "        if c is None:\n            return None\n        ctl = self.controllers[c]\n",
        "        if c is None:\n            self.next_job += 1\n            return None\n        ctl = self.controllers[c]\n"),
    "tasks assigned by another cluster's controller": (
        "        ctl = self.controllers[c]\n        local = ctl.add_job(D)\n",
        "        ctl = self.controllers[0]\n        local = ctl.add_job(D)\n"),
    "a cluster's book counts every job": (
        "            if self.jobs[j][0] == c:\n                total += self.jobs[j][2]",
        "            if True:\n                total += self.jobs[j][2]"),
    "cluster with the most free time": (
        "return min(ok)[1] if ok else None", "return max(ok)[1] if ok else None"),
    "cluster fit strict": ("ok = [(f, i) for i, f in enumerate(free) if f >= demand]",
                           "ok = [(f, i) for i, f in enumerate(free) if f > demand]"),
}

PIN_NAMES = [n for n in dir(T) if n.startswith("test_")]


def load(src: str):
    m = types.ModuleType("scheduler_copy")
    exec(compile(src, "scheduler_copy.py", "exec"), m.__dict__)
    return m


def run_pins(mod) -> list:
    """Names of the pins that fail against the given copy of the oracle."""
    saved = {k: getattr(T, k) for k in ("SchedulerOracle", "PMasterOracle", "iteration_duration", "loss",
                                        "LOSS_LIMIT_DEFAULT")}
    failed = []

    def too_long(signum, frame):
        raise TimeoutError("pin did not end")

    previous = signal.signal(signal.SIGALRM, too_long)
    try:
        for k in saved:
            setattr(T, k, getattr(mod, k))
        for name in PIN_NAMES:
            try:
                signal.setitimer(signal.ITIMER_REAL, 2.0)   # a mistake may also make a loop endless
                getattr(T, name)()
            except Exception:   # a wrong answer, a crash or no end: either way the mistake shows
                failed.append(name)
            finally:
                signal.setitimer(signal.ITIMER_REAL, 0)
    finally:
        signal.signal(signal.SIGALRM, previous)
        for k, v in saved.items():
            setattr(T, k, v)
    return failed


def test_unmutated_copy_passes_every_pin():
    assert run_pins(load(SRC)) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name):
    old, new = MUTANTS[name]
    assert SRC.count(old) == 1, f"mutation site not unique for {name!r}"
    failed = run_pins(load(SRC.replace(old, new)))
    assert failed, f"no pin notices: {name}"
