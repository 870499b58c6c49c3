"""Host logic of the library on the CPU (planning context: no device is
touched): block layout, wave packing, push state, validation, planning."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from paper_2204_03211_amd import ParameterService, PsError, WaveList, load_library
from paper_2204_03211_amd.binding import Config

CAP = 1 << 20
FAKE = 256 * 4096   # a 256-byte aligned number standing in for a device address


def reg(svc, layers, W=2):
    return svc.register_job(layers, W, 0.1, 0.9, 1e-4)


@pytest.mark.parametrize("model", ["mlp", "alexnet", "resnet50", "vgg16", "bert_base", "awd_lm"])
def test_layout_matches_oracle_split(orc, model):
    s = wl.job_config(model)
    svc = ParameterService(None)
    job, nb = reg(svc, s.layer_numel, s.W)
    want = orc.split_layers(s.layer_numel, CAP)
    assert nb == len(want) == svc.job_n_blocks(job)
    flat = 0
    prev_layer = -1
    for b, (layer, off, n) in enumerate(want):
        i = svc.job_block_info(job, b)
        assert (i.layer, i.layer_offset, i.numel, i.W) == (layer, off, n, s.W)
        if layer != prev_layer:
            flat = -(-flat // 64) * 64            # each layer starts 256-byte aligned
            layer_base, prev_layer = flat, layer
            flat += s.layer_numel[layer]
        assert i.flat_offset == layer_base + off and i.flat_offset % 4 == 0
        assert i.small_path == (1 if n <= 4096 else 0)
    assert svc.job_flat_numel(job) == -(-flat // 64) * 64
    assert ParameterService.job_arena_bytes(s.layer_numel) == 8 * svc.job_flat_numel(job)


def test_layout_random_caps_match_oracle(orc):
    rng = np.random.default_rng(0)
    for _ in range(30):
        layers = [int(x) for x in rng.integers(1, 9000, size=rng.integers(1, 9))]
        cap_bytes = int(rng.integers(1, 40)) * 256
        svc = ParameterService(None, max_block_bytes=cap_bytes)
        job, nb = reg(svc, layers)
        want = orc.split_layers(layers, cap_bytes // 4)
        got = [svc.job_block_info(job, b) for b in range(nb)]
        assert [(i.layer, i.layer_offset, i.numel) for i in got] == want
        ends = sorted((i.flat_offset, i.flat_offset + i.numel) for i in got)
        assert all(a[1] <= b[0] for a, b in zip(ends, ends[1:]))    # shards never overlap


def test_pack_wave_matches_oracle_on_the_twelve_job_wave(orc):
    specs = wl.packed_wave_jobs(42)
    svc = ParameterService(None)
    jobs = [reg(svc, s.layer_numel, s.W)[0] for s in specs]
    ojobs = []
    for s in specs:
        o = orc.OracleJob.__new__(orc.OracleJob)
        o.blocks = orc.split_layers(s.layer_numel, CAP)
        o.arrival = (lambda o=o: orc.arrival_order([b[0] for b in o.blocks]))
        ojobs.append(o)
    wave = svc.pack_wave(jobs)
    assert wave.tolist() == [(jobs[j], b) for j, b in orc.pack_wave(ojobs)]
    assert len(wave) == 1743
    # a subset of jobs, listed in another order: ties follow the listing order
    sub = [jobs[5], jobs[0], jobs[11]]
    got = svc.pack_wave(sub).tolist()
    want = [(sub[j], b) for j, b in orc.pack_wave([ojobs[5], ojobs[0], ojobs[11]])]
    assert got == want


def test_pack_wave_errors_and_capacity():
    svc = ParameterService(None)
    a, _ = reg(svc, [10, 5000])
    L = load_library()
    from paper_2204_03211_amd.binding import BlockRef
    need = C.c_int64()
    ja = (C.c_int32 * 2)(a, a)
    out = (BlockRef * 1)()
    assert L.ps_pack_wave(svc.ctx, ja, 1, out, 1, C.byref(need)) == -12 and need.value == 2
    assert L.ps_pack_wave(svc.ctx, ja, 2, out, 1, C.byref(need)) == -7      # job listed twice
    ja[1] = 99
    assert L.ps_pack_wave(svc.ctx, ja, 2, out, 1, C.byref(need)) == -2
    assert svc.pack_wave([]).tolist() == []


def test_push_state_machine():
    svc = ParameterService(None)
    job, nb = reg(svc, [5000, 10], W=3)
    cases = [
        (lambda: svc.push(job, 0, 3, FAKE), "PS_ERR_BAD_WORKER"),
        (lambda: svc.push(job, 0, -1, FAKE), "PS_ERR_BAD_WORKER"),
        (lambda: svc.push(job, 2, 0, FAKE), "PS_ERR_BAD_BLOCK"),
        (lambda: svc.push(job + 1, 0, 0, FAKE), "PS_ERR_BAD_JOB"),
        (lambda: svc.push(job, 0, 0, FAKE + 4), "PS_ERR_ALIGN"),
        (lambda: svc.push(job, 0, 0, 0), "PS_ERR_ARG"),
        (lambda: svc.push_flat(job, 0, FAKE + 16), "PS_ERR_ALIGN"),
    ]
    for fn, name in cases:
        with pytest.raises(PsError) as ei:
            fn()
        assert ei.value.name == name
    svc.push(job, 0, 1, FAKE)
    assert svc.job_block_info(job, 0).push_mask == 0b010
    with pytest.raises(PsError) as ei:
        svc.push(job, 0, 1, FAKE)
    assert ei.value.name == "PS_ERR_DUP_PUSH"
    with pytest.raises(PsError) as ei:
        svc.push_flat(job, 1, FAKE)                 # block 0 already has worker 1: nothing marked
    assert ei.value.name == "PS_ERR_DUP_PUSH"
    assert svc.job_block_info(job, 1).push_mask == 0
    svc.push_flat(job, 0, FAKE)
    svc.push_flat(job, 2, FAKE)
    assert svc.job_block_info(job, 0).push_mask == 0b111
    assert svc.job_block_info(job, 1).push_mask == 0b101
    wave = svc.pack_wave([job])
    with pytest.raises(PsError) as ei:
        svc.plan_wave(wave)                          # block 1 lacks worker 1
    assert ei.value.name == "PS_ERR_NOT_READY"
    svc.push(job, 1, 1, FAKE)
    assert svc.plan_wave(wave).n_blocks == 2
    with pytest.raises(PsError) as ei:
        svc.aggregate(wave)
    assert ei.value.name == "PS_ERR_NO_DEVICE"
    assert svc.job_block_info(job, 0).push_mask == 0b111   # refused call consumed nothing


def test_plan_validation_and_counts():
    specs = wl.packed_wave_jobs(42)
    svc = ParameterService(None)
    jobs = [reg(svc, s.layer_numel, s.W)[0] for s in specs]
    for j, s in zip(jobs, specs):
        for w in range(s.W):
            svc.push_flat(j, w, FAKE)
    wave = svc.pack_wave(jobs)
    st = svc.plan_wave(wave)
    sizes = [(svc.job_block_info(j, b).numel, specs[jobs.index(j)].W) for j, b in wave.tolist()]
    assert st.n_blocks == 1743 and st.n_params == 900_022_044
    assert st.algorithmic_bytes == sum((4 * W + 16) * n for n, W in sizes)
    assert st.n_large_tiles == sum(-(-n // 4096) for n, _ in sizes if n > 4096)
    small = [n for n, _ in sizes if n <= 4096]
    assert st.n_small_blocks == len(small) and st.small_params == sum(small)
    quads = sum(-(-n // 4) for n in small)
    assert -(-quads // 2048) <= st.n_small_bins <= len(small)
    refs = wave.tolist()
    for bad, name in [(refs + [refs[3]], "PS_ERR_DUP_BLOCK"), ([(99, 0)], "PS_ERR_BAD_JOB"),
                      ([(jobs[0], 10_000)], "PS_ERR_BAD_BLOCK"), ([(jobs[0], -1)], "PS_ERR_BAD_BLOCK")]:
        with pytest.raises(PsError) as ei:
            svc.plan_wave(WaveList(bad))
        assert ei.value.name == name
    assert svc.plan_wave(WaveList([])).n_blocks == 0


def test_argument_errors_and_unregister():
    L = load_library()
    ctx = C.c_void_p()
    for cfg in (Config(1000, 0, 0, None, 0, 0, 0), Config(0, 5000, 0, None, 0, 0, 0),
                Config(0, 0, 8, None, 0, 0, 0), Config(0, 0, 0, 128, 1 << 20, 0, 0),
                Config(2 << 30, 0, 0, None, 0, 0, 0), Config(0, 0, 0, None, 0, 0, 2001)):
        assert L.ps_create(C.byref(cfg), C.byref(ctx)) == -1
    svc = ParameterService(None)
    for layers, W, lr in [([0], 2, 0.1), ([10], 0, 0.1), ([10], 33, 0.1), ([], 2, 0.1),
                          ([10], 2, float("nan")), ([10], 2, float("inf"))]:
        with pytest.raises(PsError) as ei:
            svc.register_job(layers, W, lr, 0.9, 0.0)
        assert ei.value.name == "PS_ERR_ARG"
    a, _ = reg(svc, [100])
    b, _ = reg(svc, [100], W=32)
    assert svc.job_block_info(b, 0).W == 32
    svc.unregister_job(a)
    with pytest.raises(PsError) as ei:
        svc.job_block_info(a, 0)
    assert ei.value.name == "PS_ERR_BAD_JOB"
    with pytest.raises(PsError):
        svc.unregister_job(a)
    assert svc.job_n_blocks(b) == 1
    assert load_library().ps_strerror(-6).decode().startswith("block has not")


def test_split_ready_and_late_admission():
    """Late requests (Section 3.3.1, "Handling Outliers"): the wave takes the
    blocks whose pushes are complete; a late block joins the current cycle only
    if the time left after the work still scheduled covers it."""
    from paper_2204_03211_amd import Scheduler
    svc = ParameterService(None)
    job, nb = reg(svc, [5000, 10, 300], W=2)
    wave = svc.pack_wave([job])
    svc.push_flat(job, 0, FAKE)
    svc.push(job, 0, 1, FAKE)
    svc.push(job, 2, 1, FAKE)                     # block 1 still lacks worker 1
    ready, late = svc.split_ready(wave)
    assert ready.tolist() == [(job, 2), (job, 0)] and late.tolist() == [(job, 1)]
    assert svc.plan_wave(ready).n_blocks == 2
    with pytest.raises(PsError) as ei:
        svc.plan_wave(wave)
    assert ei.value.name == "PS_ERR_NOT_READY"
    # cycle 12 ms, 7 ms gone, 3 ms of scheduled work left: a 2 ms straggler fits, a 2.5 ms one waits
    assert Scheduler.admit_late(12.0, 7.0, 3.0, 2.0)
    assert not Scheduler.admit_late(12.0, 7.0, 3.0, 2.5)
    svc.push(job, 1, 1, FAKE)
    ready, late = svc.split_ready(wave)
    assert len(ready) == 3 and len(late) == 0
    for bad, name in [(wave.tolist() + [(job, 0)], "PS_ERR_DUP_BLOCK"), ([(job, 9)], "PS_ERR_BAD_BLOCK")]:
        with pytest.raises(PsError) as ei:
            svc.split_ready(WaveList(bad))
        assert ei.value.name == name


def test_ownership_states_on_the_host():
    """Migration bookkeeping without a device: announce / cancel, what each state
    refuses, and a shadow registration that owns nothing."""
    from paper_2204_03211_amd import OWNER_ELSEWHERE, OWNER_HERE, OWNER_LEAVING
    a, b = ParameterService(None), ParameterService(None)
    ja, nb = reg(a, [5000, 10], W=2)
    jb, nb2 = b.register_shadow_job([5000, 10], 2, 0.1, 0.9, 1e-4)
    assert nb == nb2 == 2
    assert [b.job_block_info(jb, k).owner for k in range(2)] == [OWNER_ELSEWHERE] * 2
    assert b.pack_wave([jb]).tolist() == []                  # nothing to aggregate there
    with pytest.raises(PsError) as ei:
        b.push(jb, 0, 0, FAKE)
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    with pytest.raises(PsError) as ei:
        b.pull(jb, 0)                                        # the owner answers pulls, not a shadow
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    a.push(ja, 0, 0, FAKE)
    with pytest.raises(PsError) as ei:
        a.migrate_begin(ja, 0)                               # a push of the coming round is in
    assert ei.value.name == "PS_ERR_BUSY"
    a.migrate_begin(ja, 1)
    assert a.job_block_info(ja, 1).owner == OWNER_LEAVING
    with pytest.raises(PsError) as ei:
        a.push(ja, 1, 0, FAKE)
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    assert a.pack_wave([ja]).tolist() == [(ja, 0)]
    with pytest.raises(PsError) as ei:
        a.plan_wave(WaveList([(ja, 1)]))
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    with pytest.raises(PsError) as ei:
        a.migrate_begin(ja, 1)
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    a.push_flat(ja, 1, FAKE)                                  # skips the leaving block
    assert a.job_block_info(ja, 1).push_mask == 0 and a.job_block_info(ja, 0).push_mask == 0b11
    with pytest.raises(PsError) as ei:
        a.migrate_copy(ja, 1, b, jb)                          # no device behind these contexts
    assert ei.value.name == "PS_ERR_NO_DEVICE"
    a.migrate_cancel(ja, 1)
    assert a.job_block_info(ja, 1).owner == OWNER_HERE
    with pytest.raises(PsError):
        a.migrate_cancel(ja, 1)


def test_batched_migration_checks_everything_before_anything_moves():
    a, b = ParameterService(None, max_block_bytes=1024), ParameterService(None, max_block_bytes=1024)
    ja, nb = reg(a, [1000, 10, 300], W=2)                     # 4 + 1 + 2 blocks
    jb, _ = b.register_shadow_job([1000, 10, 300], 2, 0.1, 0.9, 1e-4)
    assert nb == 7
    a.migrate_many(ja, [], b, jb)                            # nothing to do is fine
    for bad, name in (([0, 7], "PS_ERR_BAD_BLOCK"), ([1, 2, 1], "PS_ERR_DUP_BLOCK"), ([-1], "PS_ERR_BAD_BLOCK")):
        with pytest.raises(PsError) as ei:
            a.migrate_many(ja, bad, b, jb)
        assert ei.value.name == name
    a.push(ja, 3, 1, FAKE)
    with pytest.raises(PsError) as ei:
        a.migrate_many(ja, [2, 3], b, jb)                    # block 3 has a push pending
    assert ei.value.name == "PS_ERR_BUSY"
    with pytest.raises(PsError) as ei:
        b.migrate_many(jb, [0], a, ja)                       # b owns nothing
    assert ei.value.name == "PS_ERR_NOT_OWNER"
    a.migrate_begin(ja, 5)                                   # already announced blocks may be listed
    with pytest.raises(PsError) as ei:
        a.migrate_many(ja, [0, 1, 5], b, jb)                 # valid list, but no device behind these contexts
    assert ei.value.name == "PS_ERR_NO_DEVICE"
    from paper_2204_03211_amd import OWNER_HERE, OWNER_LEAVING
    assert [a.job_block_info(ja, k).owner for k in range(7)] == [OWNER_HERE] * 5 + [OWNER_LEAVING, OWNER_HERE]
    # a shadow with another block size or other layers is not the same job
    c = ParameterService(None, max_block_bytes=2048)
    jc, _ = c.register_shadow_job([1000, 10, 300], 2, 0.1, 0.9, 1e-4)
    with pytest.raises(PsError) as ei:
        a.migrate_many(ja, [0], c, jc)
    assert ei.value.name == "PS_ERR_ARG"
    with pytest.raises(PsError) as ei:
        a.migrate_many(ja, [0], a, ja)
    assert ei.value.name == "PS_ERR_ARG"


def test_pull_copy_checks_before_it_touches_the_device():
    a, b = ParameterService(None), ParameterService(None)
    ja, _ = reg(a, [5000, 10], W=2)
    jb, _ = b.register_shadow_job([5000, 10], 2, 0.1, 0.9, 1e-4)
    for args, name in (((ja, 5, FAKE), "PS_ERR_BAD_BLOCK"), ((99, 0, FAKE), "PS_ERR_BAD_JOB"),
                       ((ja, 0, 0), "PS_ERR_ARG"), ((ja, 0, FAKE), "PS_ERR_NO_DEVICE")):
        with pytest.raises(PsError) as ei:
            a.pull_copy(*args)
        assert ei.value.name == name
    with pytest.raises(PsError) as ei:
        b.pull_copy(jb, 0, FAKE)                              # a shadow holds nothing to copy
    assert ei.value.name == "PS_ERR_NOT_OWNER"


def test_predicted_wave_time_follows_the_byte_model():
    """est_seconds = sum over launches of read/7.0e12 + written/7.0e12 + 1.4 us, plus
    5 us a wave; ps_estimate_wave reports it before any push is in."""
    svc = ParameterService(None)
    W, n = 8, 3 * (1 << 20) + 5000
    j, nb = reg(svc, [n, 100], W=W)
    wave = svc.pack_wave([j])
    with pytest.raises(PsError) as ei:
        svc.plan_wave(wave)                                   # no pushes yet
    assert ei.value.name == "PS_ERR_NOT_READY"
    st = svc.estimate_wave(wave)
    large = n                                                 # the 100-element layer rides in a bin
    want = 5e-6 + st.n_launches * 1.4e-6 + (4 * W + 8) * large * 4 / 4 / 7.0e12 + 8 * large / 7.0e12
    assert st.n_launches == 1 and st.n_small_blocks == 1
    assert st.est_seconds == pytest.approx(want, rel=1e-9)
    assert svc.estimate_wave(WaveList([])).est_seconds == 0.0
    for w in range(W):
        svc.push_flat(j, w, FAKE)
    assert svc.plan_wave(wave).est_seconds == st.est_seconds
    # one block at a time: what a scheduler would use as the task's execution time
    each = [svc.estimate_wave(WaveList([(j, b)])).est_seconds for b in range(nb)]
    assert all(e > 5e-6 for e in each) and each[0] == each[1] > each[3]


def test_pushes_from_many_threads():
    """One context, one mutex: W worker threads push their gradients for every
    block at the same time; every mask ends up complete and nothing is lost."""
    import threading
    svc = ParameterService(None, max_block_bytes=1024)
    W = 16
    job, nb = reg(svc, [40_000, 3_000, 17], W=W)
    errors = []

    def worker(w):
        try:
            for b in range(nb):
                svc.push(job, b, w, FAKE + 256 * w)
        except Exception as e:          # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(w,)) for w in range(W)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    assert all(svc.job_block_info(job, b).push_mask == (1 << W) - 1 for b in range(nb))
    assert svc.plan_wave(svc.pack_wave([job])).n_blocks == nb


def test_release_spread_knob_is_validated():
    from paper_2204_03211_amd import PsError
    for ok in (-1, 0, 835, 4000):
        ParameterService(None, store_stagger_permille=ok).close()
    with pytest.raises(PsError):
        ParameterService(None, store_stagger_permille=4001)


def test_rates_of_a_planning_context_are_the_built_in_ones():
    svc = ParameterService(None)
    r = svc.rates()
    assert (r.read_bytes_per_sec, r.write_bytes_per_sec) == (7.0e12, 7.0e12)
    svc.close()


def test_noalloc_entry_point_validates_like_ps_aggregate_on_a_planning_context():
    svc = ParameterService(None)
    job, nb = reg(svc, [5000, 10], W=2)
    wave = svc.pack_wave([job])
    with pytest.raises(PsError) as ei:
        svc.aggregate_noalloc(wave)
    assert ei.value.name == "PS_ERR_NOT_READY"
    for w in range(2):
        svc.push_flat(job, w, FAKE)
    with pytest.raises(PsError) as ei:
        svc.aggregate_noalloc(WaveList(wave.tolist() + wave.tolist()[:1]))
    assert ei.value.name == "PS_ERR_DUP_BLOCK"
    with pytest.raises(PsError) as ei:
        svc.aggregate_noalloc(wave)
    assert ei.value.name == "PS_ERR_NO_DEVICE"          # valid list, but nothing to run it on
    svc.aggregate_noalloc(WaveList([]))                  # empty list: no-op
    assert svc.job_block_info(job, 0).round == 0 and svc.job_block_info(job, 0).push_mask == 3
    svc.close()
