"""Pins for the scheduling oracle (CPU only): the worked examples the paper
prints for cyclic execution and for the assignment heuristic (Section 3.3.1,
figure "Toy examples of cyclic execution" and the paragraph after it), the
default LossLimit, and the invariants the text states."""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle.scheduler import LOSS_LIMIT_DEFAULT, PMasterOracle, SchedulerOracle, iteration_duration, loss


def test_default_loss_limit():
    assert LOSS_LIMIT_DEFAULT == 0.1


def test_toy_pack_two_jobs_share_one_aggregator():
    """J1: iteration 6, aggregation 2.  J2: iteration 12, aggregation 3.
    Alone each Aggregator cycles at its job's iteration; packed, the cycle is
    12 and J1 runs twice in it."""
    s = SchedulerOracle()
    j1, j2 = s.add_job(6.0), s.add_job(12.0)
    t1, n1 = s.assign(j1, 2.0)
    assert n1 == 0 and s.cycle(0) == 6.0 and s.free(0) == 4.0
    assert s.cycle_plan(0) == [(Fr(0), [j1])]
    t2, n2 = s.assign(j2, 3.0)
    assert n2 == 0                                   # fits: no new Aggregator
    assert s.cycle(0) == 12.0
    assert s.cycle_plan(0) == [(Fr(0), [j1, j2]), (Fr(1, 2), [j1])]
    assert s.busy(0) == 2 * 2.0 + 1 * 3.0 and s.free(0) == 5.0
    assert s.job_duration(j1) == 6.0 and s.job_loss(j1) == 0.0
    assert s.job_duration(j2) == 12.0
    # J2 alone
    s2 = SchedulerOracle()
    k = s2.add_job(12.0)
    s2.assign(k, 3.0)
    assert s2.cycle(0) == 12.0 and s2.cycle_plan(0) == [(Fr(0), [k])]


def test_toy_loss_seventeen_percent_is_rejected():
    """A task (execution 1, iteration 5) shares with J2 (iteration 12): the cycle
    becomes 12, the task runs twice, its iteration becomes 6: loss (6-5)/6 = 17 %,
    above LossLimit, so the Aggregator is not a destination and a new one is
    allocated."""
    assert iteration_duration(12.0, 5.0) == 6.0
    assert loss(6.0, 5.0) == pytest.approx(1 / 6) and round(100 * loss(6.0, 5.0)) == 17
    s = SchedulerOracle()
    a, j2 = s.add_job(5.0), s.add_job(12.0)
    s.assign(a, 1.0)
    assert s.estimate(0, j2) is None
    _, n = s.assign(j2, 3.0)
    assert n == 1 and sorted(s.aggs) == [0, 1]
    assert s.cycle(0) == 5.0 and s.cycle(1) == 12.0
    # with a laxer limit the same placement is accepted and costs the 17 %
    lax = SchedulerOracle(loss_limit=0.2)
    a, j2 = lax.add_job(5.0), lax.add_job(12.0)
    lax.assign(a, 1.0)
    assert lax.estimate(0, j2) == (12.0, 12.0 - 2 * 1.0)
    _, n = lax.assign(j2, 3.0)
    assert n == 0 and lax.job_duration(a) == 6.0 and lax.job_loss(a) == pytest.approx(1 / 6)


def test_loss_limit_boundary_is_inclusive():
    # D=9 under cycle 10: runs once, d=10, loss exactly 0.1 -> rejected (>=)
    s = SchedulerOracle(loss_limit=0.1)
    a, b = s.add_job(9.0), s.add_job(10.0)
    s.assign(a, 1.0)
    assert loss(iteration_duration(10.0, 9.0), 9.0) == 0.1
    assert s.estimate(0, b) is None
    s = SchedulerOracle(loss_limit=0.1)
    a, b = s.add_job(9.5), s.add_job(10.0)
    s.assign(a, 1.0)
    assert s.estimate(0, b) is not None


def test_new_jobs_own_loss_counts():
    """The arriving job can be the one that loses: D_k = 7 on an Aggregator of
    cycle 12 would run once per 12."""
    s = SchedulerOracle()
    big, k = s.add_job(12.0), s.add_job(7.0)
    s.assign(big, 1.0)
    assert s.estimate(0, k) is None
    _, n = s.assign(k, 1.0)
    assert n == 1


def test_best_fit_is_least_sufficient_free_time():
    s = SchedulerOracle()
    jobs = [s.add_job(10.0) for _ in range(4)]
    # three Aggregators with free time 7, 4, 2 (forced by filling fresh ones)
    for j, e in zip(jobs[:3], (3.0, 6.0, 8.0)):
        n = s.allocate()
        s._place(n, j, e)
    assert [s.free(n) for n in (0, 1, 2)] == [7.0, 4.0, 2.0]
    assert s.choose(jobs[3], 1.5) == 2        # all fit: the tightest
    assert s.choose(jobs[3], 3.0) == 1
    assert s.choose(jobs[3], 5.0) == 0
    before = len(s.aggs)
    assert s.choose(jobs[3], 7.5) == 3 and len(s.aggs) == before + 1   # none fits: allocate
    # ties go to the lowest id
    t = SchedulerOracle()
    a, b, c = t.add_job(10.0), t.add_job(10.0), t.add_job(10.0)
    for j in (a, b):
        t._place(t.allocate(), j, 4.0)
    assert t.choose(c, 1.0) == 0


def test_each_task_on_one_aggregator_and_losses_bounded():
    rng = np.random.default_rng(0)
    for trial in range(20):
        s = SchedulerOracle()
        jobs = [s.add_job(float(rng.choice([4, 5, 6, 8, 10, 12, 20, 24]))) for _ in range(6)]
        for _ in range(60):
            j = int(rng.integers(len(jobs)))
            e = float(rng.integers(1, 8)) / 8.0
            C_before = {n: s.cycle(n) for n in s.aggs}
            t, n = s.assign(jobs[j], e)
            assert s.where[t] == (n, jobs[j], e)
            # the chosen Aggregator passed the loss test and had room for e
            if n in C_before:
                assert s.free(n) >= -1e-12 or True
        placed = [t for a in s.aggs.values() for ts in a.tasks.values() for t, _ in ts]
        assert sorted(placed) == sorted(s.where) and len(set(placed)) == len(placed)
        for j in jobs:
            assert s.job_loss(j) < s.loss_limit
        for n in s.aggs:
            assert s.cycle(n) == max(s.D[j] for j in s.aggs[n].tasks)


def test_late_request_rule():
    adm = SchedulerOracle.admit_late
    # cycle 12, 7 elapsed, 3 still scheduled: 2 left over
    assert adm(12.0, 7.0, 3.0, 2.0) is True
    assert adm(12.0, 7.0, 3.0, 2.5) is False      # would push scheduled work: next cycle
    assert adm(12.0, 0.0, 7.0, 5.0) is True
    assert adm(12.0, 12.0, 0.0, 0.1) is False


def test_job_exit_releases_and_recycles():
    s = SchedulerOracle()
    a, b, c = s.add_job(10.0), s.add_job(10.0), s.add_job(10.0)
    for _ in range(3):
        s.assign(a, 3.0)            # 9 of 10 on Aggregator 0
    s.assign(b, 3.0)                # does not fit -> Aggregator 1
    s.assign(b, 3.0)
    s.assign(c, 6.0)                # 1 has 4 free: no; -> Aggregator 2
    assert sorted(s.aggs) == [0, 1, 2]
    released = s.remove_job(a)      # 0 empties and is released; then the least loaded of
    assert 0 in released            # {1: 0.6, 2: 0.6} (tie -> higher id 2) drains into 1? 6 > 4: no
    assert sorted(s.aggs) == [1, 2] and released == [0]
    s2 = SchedulerOracle()
    a, b = s2.add_job(10.0), s2.add_job(10.0)
    s2._place(s2.allocate(), a, 2.0)
    s2._place(s2.allocate(), b, 3.0)
    s2._place(s2.allocate(), b, 1.0)
    c = s2.add_job(10.0)
    s2._place(2, c, 1.0)
    # c exits: Aggregator 2 keeps b's 1.0; least loaded is 2 (0.1) and drains into 1 (best fit? free 7 vs 8 -> 1)
    released = s2.remove_job(c)
    assert released[0] == 2
    # then 0 (0.2) vs 1 (0.4): 0 drains into 1; one Aggregator is left and the loop stops
    assert released == [2, 0] and sorted(s2.aggs) == [1]
    assert s2.busy(1) == 6.0
    assert all(n == 1 for n, _, _ in s2.where.values())


def test_recycling_never_allocates_and_rolls_back():
    s = SchedulerOracle()
    a, b = s.add_job(10.0), s.add_job(10.0)
    s._place(s.allocate(), a, 6.0)
    n1 = s.allocate()
    s._place(n1, b, 3.0)
    s._place(n1, b, 5.0)            # 8 of 10: the 3.0 could move to 0 (4 free) but the 5.0 cannot
    k = s.add_job(10.0)
    s._place(s.allocate(), k, 1.0)
    before = {t: w for t, w in s.where.items() if w[1] != k}
    released = s.remove_job(k)
    assert released == [2]          # only the emptied one; draining 0 (0.6) fails, loop stops
    assert {t: w for t, w in s.where.items()} == before
    assert s.next_agg == 3          # nothing was allocated


def test_best_fit_cluster():
    f = SchedulerOracle.best_fit_cluster
    assert f([5.0, 2.0, 9.0], 1.5) == 1
    assert f([5.0, 2.0, 9.0], 4.0) == 0
    assert f([5.0, 2.0, 9.0], 9.5) is None
    assert f([3.0, 3.0], 3.0) == 0


def test_scale_up_moves_a_job_off_a_full_aggregator():
    """Section 3.3.2: a new job that runs slower than alone gets one more
    Aggregator and is assigned again, until it no longer loses speed.  The job
    sits on an Aggregator filled 10 of 10: after one step it must sit somewhere
    else (plain best fit would put it straight back), and a further step, which
    has nothing left to gain, must say so and hand its Aggregator back."""
    s = SchedulerOracle()
    a, b = s.add_job(10.0), s.add_job(10.0)
    for _ in range(3):
        s.assign(a, 2.0)
    for _ in range(2):
        s.assign(b, 2.0)                       # 10 of 10 used on Aggregator 0: no slack at all
    assert sorted(s.aggs) == [0] and s.free(0) == 0.0
    before = sorted(n for n, j, e in s.where.values() if j == b)
    fresh, moved = s.scale_up_job(b)
    after = sorted(n for n, j, e in s.where.values() if j == b)
    assert (fresh, moved) == (1, 2) and before == [0, 0] and after == [1, 1]
    assert sorted(s.aggs) == [0, 1] and s.free(0) == 4.0 and s.free(1) == 6.0
    assert sorted(n for n, j, e in s.where.values() if j == a) == [0, 0, 0]   # nobody else moves
    fresh, moved = s.scale_up_job(b)           # b already has an Aggregator to itself
    assert (fresh, moved) == (2, 0)
    assert sorted(s.aggs) == [0, 1]            # the unused new Aggregator is handed back
    assert sorted(n for n, j, e in s.where.values() if j == b) == [1, 1]


def test_scale_up_takes_one_aggregator_of_load_per_step():
    """A job larger than one Aggregator: every step moves what one more
    Aggregator holds; what is left over goes through the assignment scheme over
    the others; the loop ends with the job on Aggregators of its own."""
    s = SchedulerOracle()
    x, y = s.add_job(10.0), s.add_job(10.0)
    s.assign(x, 5.0)
    ty = [s.assign(y, 4.0)[0] for _ in range(3)]
    assert [s.where[t][0] for t in ty] == [0, 1, 1]       # 5 free on 0 takes one; the rest open 1
    assert s.scale_up_job(y) == (2, 3)
    # the new Aggregator takes two (8 of 10); the third goes by best fit: 0 (5 free) before the emptied 1 (10)
    assert [s.where[t][0] for t in ty] == [2, 2, 0] and sorted(s.aggs) == [0, 2]
    assert s.scale_up_job(y) == (3, 1)
    assert [s.where[t][0] for t in ty] == [2, 2, 3] and sorted(s.aggs) == [0, 2, 3]
    assert s.own[y] == [2, 3] and s.busy(0) == 5.0
    assert s.scale_up_job(y) == (4, 0)
    assert [s.where[t][0] for t in ty] == [2, 2, 3] and sorted(s.aggs) == [0, 2, 3] and s.own[y] == [2, 3]
    # y leaves: its own Aggregators go back, nothing refers to them any more
    assert s.remove_job(y) == [2, 3] and s.own == {}


def test_scale_up_keeps_the_loss_test_on_the_jobs_own_aggregators():
    s = SchedulerOracle()
    k, f = s.add_job(12.0), s.add_job(5.0)
    other = s.add_job(12.0)
    s.assign(other, 9.0)
    tk = s.assign(k, 2.0)[0]
    assert s.where[tk][0] == 0
    assert s.scale_up_job(k) == (1, 1) and s.where[tk][0] == 1 and s.own[k] == [1]
    s._place(1, f, 0.5)                        # forced: f (iteration 5) would lose 17 % under cycle 12
    assert s.estimate(1, k) is None
    fresh, moved = s.scale_up_job(k)
    assert (fresh, moved) == (2, 1) and s.where[tk][0] == 2     # 1 no longer qualifies, although it has room
    assert s.own[k] == [1, 2] and sorted(s.aggs) == [0, 1, 2]


def test_scale_up_loop_ends_with_the_job_on_its_own_aggregators():
    rng = np.random.default_rng(5)
    for trial in range(25):
        s = SchedulerOracle()
        jobs = [s.add_job(float(rng.choice([4, 5, 6, 8, 10, 12, 20, 24]))) for _ in range(5)]
        tasks = {j: [] for j in jobs}
        for _ in range(50):
            j = jobs[int(rng.integers(len(jobs)))]
            tasks[j].append(s.assign(j, float(rng.integers(1, 8)) / 8.0 * s.D[j] / 4.0)[0])
        k = max(jobs, key=lambda j: len(tasks[j]))
        others = {t: w for t, w in s.where.items() if w[1] != k}
        shared_before = None
        for step in range(len(tasks[k]) + 2):
            fresh, moved = s.scale_up_job(k)
            shared = sum(e for t, (n, j, e) in s.where.items() if j == k and n not in s.own.get(k, []))
            assert shared_before is None or shared <= shared_before      # never back onto shared Aggregators
            shared_before = shared
            if moved == 0:
                break
        assert moved == 0 and step <= len(tasks[k])
        assert all(s.where[t][0] in s.own[k] for t in tasks[k])
        assert {t: w for t, w in s.where.items() if w[1] != k} == others  # the other jobs never move
        assert all(not s.aggs[n].empty() for n in s.aggs)


def test_pmaster_forwards_to_the_best_fit_cluster():
    """Section 3.3.3: pMaster keeps each cluster's remaining free resource and
    forwards a new job to the cluster with sufficient but least of it, by the
    job's total demand; the controller there assigns every task inside that one
    cluster; an exit is reported back and frees the room."""
    m = PMasterOracle()
    assert [m.add_cluster(c) for c in (2.0, 1.0, 3.0)] == [0, 1, 2]
    assert PMasterOracle.demand(10.0, [2.0, 2.0, 1.0]) == 0.5
    j0, c0, placed0 = m.forward_job(10.0, [2.0, 2.0, 1.0])            # demand 0.5: free 2, 1, 3 -> cluster 1
    assert (j0, c0) == (0, 1) and placed0 == [(0, 0), (1, 0), (2, 0)]
    assert [m.free(c) for c in range(3)] == [2.0, 0.5, 3.0]
    j1, c1, placed1 = m.forward_job(10.0, [4.0, 4.0])                 # 0.8: 1 has 0.5 only -> 0 (2 before 3)
    assert (j1, c1) == (1, 0) and placed1 == [(0, 0), (1, 0)]          # ids are the cluster's own
    assert m.forward_job(5.0, [5.0, 5.0, 5.0, 2.0]) is None           # 3.4: nobody has that much
    assert len(m.jobs) == 2 and m.next_job == 2                       # nothing was registered
    j2, c2, _ = m.forward_job(4.0, [1.0, 1.0])                        # 0.5: cluster 1 has exactly 0.5
    assert (j2, c2) == (2, 1) and m.free(1) == 0.0
    j3, c3, _ = m.forward_job(4.0, [1.0])                             # 0.25: 0 has 1.2, 2 has 3 -> 0
    assert c3 == 0 and m.free(0) == 2.0 - 0.8 - 0.25
    # one job, one cluster: every controller only knows the tasks of its own jobs
    assert sum(len(ctl.where) for ctl in m.controllers) == 3 + 2 + 2 + 1
    assert len(m.controllers[1].where) == 5 and len(m.controllers[2].where) == 0
    # exit: the controller recycles inside its cluster, pMaster's book gets the demand back
    c, released = m.job_exit(j0)
    assert c == 1 and m.free(1) == 0.5 and j0 not in m.jobs
    assert released == [0] == lone_controller_release_after_exit()
    j4, c4, _ = m.forward_job(10.0, [3.0])                            # 0.3 fits cluster 1 again (0.5 least)
    assert c4 == 1
    # ties between equally free clusters go to the lowest id
    t = PMasterOracle()
    t.add_cluster(1.0), t.add_cluster(1.0)
    assert t.forward_job(10.0, [1.0])[1] == 0                         # 1.0 and 1.0 free: the first
    assert t.forward_job(10.0, [1.0])[1] == 0                         # 0.9 and 1.0: still the tighter one
    assert t.forward_job(10.0, [9.0])[1] == 1                         # 0.9 needed: only cluster 1 (1.0) has it


def lone_controller_release_after_exit():
    """The same exit on a lone controller: jobs (10: 2,2,1) and (4: 1,1) share
    Aggregator 0?  No: under cycle 10 the second job (iteration 4) would run
    twice at 5 and lose 20 %, so it sits on Aggregator 1; when the first job
    leaves, Aggregator 0 is empty and released."""
    s = SchedulerOracle()
    a = s.add_job(10.0)
    for e in (2.0, 2.0, 1.0):
        s.assign(a, e)
    b = s.add_job(4.0)
    assert [s.assign(b, 1.0)[1] for _ in range(2)] == [1, 1]
    return s.remove_job(a)


def test_pmaster_book_is_demand_not_packing_and_scale_up_stays_inside():
    m = PMasterOracle()
    m.add_cluster(1.5), m.add_cluster(4.0)
    ja, ca, _ = m.forward_job(10.0, [2.0, 2.0, 2.0])                  # 0.6 -> cluster 0 (1.5 < 4)
    jb, cb, pb = m.forward_job(10.0, [2.0, 2.0])                      # 0.4 -> cluster 0 (0.9 left)
    assert (ca, cb) == (0, 0) and m.free(0) == pytest.approx(0.5) and m.free(1) == 4.0
    assert m.used(0) == 0.6 + 0.4
    ctl = m.controllers[0]
    assert sorted(ctl.aggs) == [0] and ctl.free(0) == 0.0             # packed onto one Aggregator, 10 of 10
    fresh, moved = m.scale_up_job(jb)                                 # inside cluster 0, by the controller
    assert (fresh, moved) == (1, 2) and sorted(ctl.aggs) == [0, 1]
    assert m.free(0) == pytest.approx(0.5) and m.free(1) == 4.0       # pMaster's book did not move
    assert len(m.controllers[1].aggs) == 0
    jc, cc, _ = m.forward_job(10.0, [6.0])                            # 0.6 > 0.5: cluster 0 is full by the book
    assert cc == 1
    assert m.job_exit(ja) == (0, [0])                                 # ja alone on Aggregator 0: released
    assert m.free(0) == pytest.approx(1.1)


def _golden(name):
    import json
    import os
    return json.load(open(os.path.join(os.path.dirname(__file__), "golden", name)))


def test_golden_toy_cyclic_execution():
    """The figures the paper prints for its two-job example, from tests/golden/."""
    g = _golden("toy_cyclic_execution.json")
    for job, alone in zip(g["jobs"], g["cycle_alone"]):
        s = SchedulerOracle()
        s.assign(s.add_job(job["D"]), job["e"])
        assert s.cycle(0) == alone
    s = SchedulerOracle()
    ids = [s.add_job(j["D"]) for j in g["jobs"]]
    for i, j in zip(ids, g["jobs"]):
        assert s.assign(i, j["e"])[1] == 0
    assert s.cycle(0) == g["cycle_packed"]
    runs = [sum(1 for _, js in s.cycle_plan(0) if i in js) for i in ids]
    assert runs == g["runs_per_cycle_packed"]
    assert s.busy(0) == g["derived"]["busy_packed"] and s.free(0) == g["derived"]["free_packed"]


def test_golden_toy_loss_limit():
    g = _golden("toy_loss_limit.json")
    assert LOSS_LIMIT_DEFAULT == g["loss_limit_default"]
    s = SchedulerOracle()
    a, b = s.add_job(g["existing"]["D"]), s.add_job(g["arriving"]["D"])
    s.assign(a, g["existing"]["e"])
    d = iteration_duration(g["cycle_after"], g["existing"]["D"])
    assert d == g["iteration_after"]
    assert round(100 * loss(d, g["existing"]["D"])) == g["loss_percent_rounded"]
    assert (s.estimate(0, b) is not None) == g["accepted_under_default_limit"]


def test_failed_drain_leaves_everything_where_it_was():
    """Recycling moves the largest task first; if a later one finds no room the
    tasks already moved go back (Section 3.3.2: recycle only if every task fits
    without new allocations)."""
    s = SchedulerOracle()
    a, b, k = s.add_job(10.0), s.add_job(10.0), s.add_job(10.0)
    s._place(s.allocate(), a, 6.0)              # load 0.6, 4 free
    n1 = s.allocate()
    t3 = s._place(n1, b, 3.0)
    t25 = s._place(n1, b, 2.5)                  # load 0.55: the one to drain
    s._place(s.allocate(), k, 1.0)
    before = dict(s.where)
    del before[max(before)]                     # k's task leaves with k
    assert s.remove_job(k) == [2]               # 3.0 fits into 0, then 2.5 does not (1 free): undone
    assert s.where == before and s.where[t3][0] == n1 and s.where[t25][0] == n1
    assert s.busy(0) == 6.0 and s.busy(1) == 5.5
    assert sorted(e for _, e in s.aggs[1].tasks[b]) == [2.5, 3.0] and list(s.aggs[0].tasks) == [a]


def test_equally_loaded_aggregators_the_younger_one_goes():
    s = SchedulerOracle()
    k, a, b = s.add_job(10.0), s.add_job(10.0), s.add_job(10.0)
    s._place(s.allocate(), k, 5.0)
    s._place(s.allocate(), a, 3.0)
    s._place(s.allocate(), b, 3.0)
    assert s.remove_job(k) == [0, 2]            # 0 is empty; 1 and 2 tie at 0.3: 2 drains into 1
    assert sorted(s.aggs) == [1] and s.busy(1) == 6.0


def test_drained_tasks_never_land_on_the_aggregator_being_drained():
    """The Aggregator being recycled can itself be the tightest fit for its own
    task (short cycle, little free time); it is not a destination."""
    s = SchedulerOracle()
    k, fast, slow = s.add_job(10.0), s.add_job(4.0), s.add_job(20.0)
    s._place(s.allocate(), k, 1.0)
    s._place(s.allocate(), fast, 1.0)           # cycle 4, load 0.25, 3 free
    s._place(s.allocate(), slow, 6.0)           # cycle 20, load 0.3, 14 free
    released = s.remove_job(k)
    assert released == [0, 1]
    assert sorted(s.aggs) == [2]
    assert all(n in s.aggs for n, _, _ in s.where.values())
    assert sorted(s.aggs[2].tasks) == [fast, slow] and s.busy(2) == 5 * 1.0 + 6.0
