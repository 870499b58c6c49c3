"""The library's scheduler against the oracle (host only, runs without a GPU):
the paper's worked examples through the C ABI, then random job arrival / task
assignment / job exit sequences compared decision by decision."""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle.scheduler import PMasterOracle, SchedulerOracle
from paper_2204_03211_amd import PMaster, PsError, Scheduler


def test_toy_examples_through_the_c_abi():
    s = Scheduler()
    j1, j2 = s.add_job(6.0), s.add_job(12.0)
    assert s.assign(j1, 2.0) == (0, 0)
    assert s.assign(j2, 3.0) == (1, 0)
    a = s.aggregator_info(0)
    assert (a.cycle, a.busy, a.free_time, a.n_jobs, a.n_tasks) == (12.0, 7.0, 5.0, 2, 2)
    assert s.cycle_plan(0) == [(Fr(0), [j1, j2]), (Fr(1, 2), [j1])]
    assert s.job_info(j1).d == 6.0 and s.job_info(j1).loss == 0.0
    t = Scheduler()
    a, b = t.add_job(5.0), t.add_job(12.0)
    t.assign(a, 1.0)
    assert t.estimate(0, b) is None                  # 17 % loss: not a destination
    assert t.assign(b, 3.0)[1] == 1
    lax = Scheduler(loss_limit=0.2)
    a, b = lax.add_job(5.0), lax.add_job(12.0)
    lax.assign(a, 1.0)
    assert lax.estimate(0, b) == (12.0, 10.0)
    assert lax.assign(b, 3.0)[1] == 0
    ji = lax.job_info(a)
    assert ji.d == 6.0 and ji.loss == pytest.approx(1 / 6) and ji.n_tasks == 1


def test_static_rules():
    assert Scheduler.admit_late(12.0, 7.0, 3.0, 2.0) and not Scheduler.admit_late(12.0, 7.0, 3.0, 2.5)
    assert Scheduler.best_fit_cluster([5.0, 2.0, 9.0], 1.5) == 1
    assert Scheduler.best_fit_cluster([5.0, 2.0, 9.0], 9.5) is None
    assert Scheduler.best_fit_cluster([], 1.0) is None


def test_errors():
    s = Scheduler()
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(PsError):
            s.add_job(bad)
    j = s.add_job(3.0)
    for fn in (lambda: s.assign(j + 1, 1.0), lambda: s.assign(j, 0.0), lambda: s.aggregator_info(0),
               lambda: s.task_info(0), lambda: s.remove_job(7)):
        with pytest.raises(PsError):
            fn()
    with pytest.raises(PsError):
        Scheduler(loss_limit=1.0)
    s.assign(j, 1.0)
    assert s.remove_job(j) == [0] and s.aggregators() == []
    with pytest.raises(PsError):
        s.assign(j, 1.0)                              # the job has left


def snapshot(o: SchedulerOracle):
    return {
        "aggs": sorted(o.aggs),
        "where": {t: (n, j, e) for t, (n, j, e) in o.where.items()},
        "info": {n: (o.cycle(n), o.busy(n), o.free(n)) for n in o.aggs},
        "plan": {n: o.cycle_plan(n) for n in o.aggs},
        "jobs": {j: (o.job_duration(j), o.job_loss(j)) for j in o.D},
    }


def compare(o: SchedulerOracle, s: Scheduler):
    snap = snapshot(o)
    assert s.aggregators() == snap["aggs"]
    for t, w in snap["where"].items():
        assert s.task_info(t) == w
    for n, (C, W, F) in snap["info"].items():
        a = s.aggregator_info(n)
        assert (a.cycle, a.busy, a.free_time) == (C, W, F)          # same doubles, same order
        assert s.cycle_plan(n) == snap["plan"][n]
    for j, (d, l) in snap["jobs"].items():
        ji = s.job_info(j)
        assert (ji.d, ji.loss) == (d, l)


@pytest.mark.parametrize("seed", range(12))
def test_random_sequences_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    limit = float(rng.choice([0.05, 0.1, 0.2, 0.34]))
    o, s = SchedulerOracle(limit), Scheduler(limit)
    durations = [3.0, 4.0, 5.0, 6.0, 7.5, 9.0, 10.0, 12.0, 0.3, 0.1, 24.0]
    live = []
    for step in range(160):
        r = rng.random()
        if r < 0.12 or not live:
            D = float(rng.choice(durations))
            jo, js = o.add_job(D), s.add_job(D)
            assert jo == js
            live.append(jo)
        elif r < 0.92:
            j = int(rng.choice(live))
            e = float(rng.integers(1, 40)) * o.D[j] / 64.0
            for n in list(o.aggs):
                assert s.estimate(n, j) == o.estimate(n, j)
            assert s.assign(j, e) == o.assign(j, e)
        elif r < 0.95:
            j = int(rng.choice(live))
            assert s.scale_up_job(j) == o.scale_up_job(j)
        else:
            j = live.pop(int(rng.integers(len(live))))
            assert s.remove_job(j) == o.remove_job(j)
        if step % 8 == 0:
            compare(o, s)
    compare(o, s)
    assert len(o.aggs) >= 1 or not live


def test_scale_up_through_the_c_abi_makes_progress_and_ends():
    """The case that used to be a no-op: a job on an Aggregator filled 10 of 10
    must sit elsewhere after one step; the loop 'while slow and moved' ends."""
    s = Scheduler()
    a, b = s.add_job(10.0), s.add_job(10.0)
    ta = [s.assign(a, 2.0)[0] for _ in range(3)]
    tb = [s.assign(b, 2.0)[0] for _ in range(2)]
    assert s.aggregators() == [0] and s.aggregator_info(0).free_time == 0.0
    assert s.scale_up_job(b) == (1, 2)
    assert [s.task_info(t)[0] for t in tb] == [1, 1] and [s.task_info(t)[0] for t in ta] == [0, 0, 0]
    steps = 1
    while True:
        fresh, moved = s.scale_up_job(b)
        steps += 1
        if moved == 0:
            break
    assert steps == 2 and s.aggregators() == [0, 1]
    with pytest.raises(PsError):
        s.scale_up_job(7)


def compare_pmaster(o: PMasterOracle, m: PMaster):
    assert m.n_clusters() == len(o.capacity)
    for c in range(len(o.capacity)):
        ci = m.cluster_info(c)
        assert (ci.capacity, ci.used, ci.free_resource) == (o.capacity[c], o.used(c), o.free(c))
        assert ci.n_jobs == sum(1 for j in o.jobs.values() if j[0] == c)
        assert ci.n_aggregators == len(o.controllers[c].aggs)
        compare(o.controllers[c], m.controller(c))
    for j, w in o.jobs.items():
        assert m.job_info(j) == w


def test_pmaster_hand_cases_through_the_c_abi():
    m = PMaster()
    assert [m.add_cluster(c) for c in (2.0, 1.0, 3.0)] == [0, 1, 2]
    assert m.forward_job(10.0, [2.0, 2.0, 1.0]) == (0, 1, [(0, 0), (1, 0), (2, 0)])   # sufficient but least
    assert m.forward_job(10.0, [4.0, 4.0]) == (1, 0, [(0, 0), (1, 0)])
    assert m.forward_job(5.0, [5.0, 5.0, 5.0, 2.0]) is None                             # none fits
    assert m.cluster_info(1).free_resource == 0.5 and m.cluster_info(1).n_jobs == 1
    assert m.job_exit(0) == (1, [0])                                                    # exit frees the room
    assert m.cluster_info(1).free_resource == 1.0 and m.cluster_info(1).n_jobs == 0
    with pytest.raises(PsError):
        m.job_exit(0)
    with pytest.raises(PsError):
        m.forward_job(10.0, [])
    with pytest.raises(PsError):
        m.forward_job(10.0, [1.0, -1.0])
    with pytest.raises(PsError):
        m.add_cluster(0.0)
    with pytest.raises(PsError):
        m.controller(9)
    assert m.forward_job(10.0, [9.0])[1] == 1                                           # 0.9 into the freed cluster


@pytest.mark.parametrize("seed", range(8))
def test_pmaster_random_sequences_match_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    limit = float(rng.choice([0.05, 0.1, 0.2]))
    o, m = PMasterOracle(limit), PMaster(limit)
    for _ in range(int(rng.integers(2, 5))):
        cap = float(rng.integers(2, 9)) / 2.0
        assert o.add_cluster(cap) == m.add_cluster(cap)
    durations = [3.0, 4.0, 5.0, 6.0, 7.5, 9.0, 10.0, 12.0, 24.0]
    live = []
    for step in range(120):
        r = rng.random()
        if r < 0.55 or not live:
            D = float(rng.choice(durations))
            es = [float(rng.integers(1, 24)) * D / 64.0 for _ in range(int(rng.integers(1, 9)))]
            got, want = m.forward_job(D, es), o.forward_job(D, es)
            assert got == want
            if want is not None:
                live.append(want[0])
        elif r < 0.75:
            j = int(rng.choice(live))
            assert m.scale_up_job(j) == o.scale_up_job(j)
        else:
            j = live.pop(int(rng.integers(len(live))))
            assert m.job_exit(j) == o.job_exit(j)
        if step % 6 == 0:
            compare_pmaster(o, m)
    compare_pmaster(o, m)
    assert sorted(o.jobs) == sorted(live)


def test_cycle_plan_refuses_an_absurd_number_of_runs_per_cycle():
    s = Scheduler(loss_limit=0.5)
    fast, slow = s.add_job(1e-4), s.add_job(10.0)
    assert s.assign(fast, 1e-6)[1] == 0 and s.assign(slow, 0.5)[1] == 0
    with pytest.raises(PsError):
        s.cycle_plan(0)                      # 100 000 runs of the fast job in one cycle
    ok = Scheduler(loss_limit=0.5)
    a, b = ok.add_job(1.0), ok.add_job(1000.0)
    ok.assign(a, 0.01), ok.assign(b, 1.0)
    plan = ok.cycle_plan(0)
    assert len(plan) == 1000 and plan[0][1] == [a, b] and all(w[1] == [a] for w in plan[1:])


def test_assignment_rate_is_job_event_scale():
    """The heuristic runs at job-event rate (Section 3.3.3: a job brings hundreds
    or thousands of model aggregations, each of which scans the Aggregators).
    The library keeps running sums per job and Aggregator, so an assignment
    costs a pass over Aggregators x jobs there, not over tasks: 40 000
    assignments over a few dozen Aggregators take well under a second, and ten
    times more tasks cost about ten times more, not a hundred."""
    import time

    def run(n_tasks):
        s = Scheduler()
        jobs = [s.add_job(float(d)) for d in (4, 5, 6, 8, 10, 12, 16, 20, 24, 30) * 4]
        t0 = time.perf_counter()
        for i in range(n_tasks):
            s.assign(jobs[i % len(jobs)], (0.05 + (i % 7) * 0.01) * 4000 / n_tasks)
        return time.perf_counter() - t0, len(s.aggregators())

    t_small, a_small = run(4000)
    t_big, a_big = run(40000)
    assert t_big < 5.0 and a_small >= 2 and a_big >= 2
    assert t_big < 40 * max(t_small, 1e-3)


def test_predicted_wave_times_as_execution_times():
    """The profiler's role (Section 3.3.1): a task's execution time comes from
    the service's own prediction of the wave, here for whole jobs at full size on
    a planning context.  VGG-16 (1.0 ms) and AlexNet (0.44 ms) share an
    Aggregator whose cycle is 1.5 ms; ResNet-50 (0.30 ms) no longer fits."""
    import workloads as wl
    from paper_2204_03211_amd import ParameterService
    svc = ParameterService(None)
    sch = Scheduler()
    placed = {}
    for name in ("vgg16", "alexnet", "resnet50"):
        s = wl.job_config(name)
        j, _ = svc.register_job(s.layer_numel, s.W, s.lr, s.momentum, s.wd)
        e_ms = svc.estimate_wave(svc.pack_wave([j])).est_seconds * 1e3
        placed[name] = (e_ms, sch.assign(sch.add_job(1.5), e_ms)[1])
    assert placed["vgg16"][0] == pytest.approx(1.0, rel=0.03)
    assert placed["alexnet"][0] == pytest.approx(0.44, rel=0.03)
    assert placed["resnet50"][0] == pytest.approx(0.30, rel=0.03)
    assert [placed[n][1] for n in ("vgg16", "alexnet", "resnet50")] == [0, 0, 1]
    svc.close()
