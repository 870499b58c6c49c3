"""ps_aggregate_noalloc (the entry point for callers that cannot allocate)
against ps_aggregate, through the C ABI: same jobs, same seeded gradients, the
same waves; parameters and momentum must be bit-identical and the telemetry
values equal, on consecutive calls of which the later ones are smaller.  The
two services are separate contexts on the one GPU; every no-alloc call shares
that GPU's static array."""
import numpy as np
import pytest
import torch

import workloads as wl
from harness import GpuService
from paper_2204_03211_amd import PsError, WaveList

pytestmark = pytest.mark.gpu


def spec(layers, W, lr=0.1, mu=0.9, wd=1e-4):
    return wl.JobSpec("synthetic", tuple(layers), W, lr, mu, wd, 1e-2, 0.05)


def assert_same(a: GpuService, b: GpuService, what: str):
    torch.cuda.synchronize()
    for ji, j in enumerate(a.jobs):
        pa, va = a.svc.pull_flat(j)
        pb, vb = b.svc.pull_flat(b.jobs[ji])
        assert torch.equal(pa.view(torch.int32), pb.view(torch.int32)), (what, ji, "parameters")
        assert torch.equal(va.view(torch.int32), vb.view(torch.int32)), (what, ji, "momentum")
        for blk in range(a.svc.job_n_blocks(j)):
            sa, sb = a.svc.telemetry(j, blk), b.svc.telemetry(b.jobs[ji], blk)
            assert (sa.round, sa.grad_norm2) == (sb.round, sb.grad_norm2), (what, ji, blk)


def test_noalloc_entry_point_matches_ps_aggregate():
    specs = [spec([300_000, 100, 4097, 7], 4), spec([64, 64, 90_000, 5000], 16, lr=0.01, mu=0.5),
             spec([123_457], 3, lr=0.05, mu=0.0, wd=0.0), spec([33, 2000, 50_001], 2)]
    ref = GpuService(specs, 17, max_block_bytes=256 * 1024)
    alt = GpuService(specs, 17, max_block_bytes=256 * 1024)
    full = ref.wave()
    refs = full.tolist()
    assert refs == alt.wave().tolist()
    # the second list is smaller than the first (one job's blocks only), the third smaller again
    one_job = [r for r in refs if r[0] == ref.jobs[1]]
    few = one_job[: max(2, len(one_job) // 3)]
    plan = [refs, one_job, few, refs, refs]
    for r, lst in enumerate(plan):
        for g in (ref, alt):
            g.fill_grads(r)
            for (j, b) in lst:
                ji = g.jobs.index(j)
                _, _, n, flat = g.blocks[ji][b]
                for w in range(specs[ji].W):
                    g.svc.push(j, b, w, g.grads[ji][w][flat:flat + n])
        ref.svc.aggregate(WaveList(lst))
        alt.svc.aggregate_noalloc(WaveList(lst))
        assert_same(ref, alt, f"call {r} ({len(lst)} blocks)")
    # two contexts taking turns on the one array, on different streams, unsynchronised
    third = GpuService(specs, 17, max_block_bytes=256 * 1024)
    side = torch.cuda.Stream()
    for r in range(len(plan), len(plan) + 3):
        for g in (ref, alt, third):
            g.fill_grads(r)
            g.push_all()
        torch.cuda.synchronize()
        ref.svc.aggregate(full)
        alt.svc.aggregate_noalloc(full)
        with torch.cuda.stream(side):
            third.svc.aggregate_noalloc(full, stream=side)
        assert_same(ref, alt, f"shared array, call {r}")
    # `third` ran only these three rounds: a context that did the same through ps_aggregate
    fresh = GpuService(specs, 17, max_block_bytes=256 * 1024)
    for r in range(len(plan), len(plan) + 3):
        fresh.fill_grads(r)
        fresh.push_all()
        fresh.svc.aggregate(full)
    assert_same(fresh, third, "third context")
    for g in (ref, alt, third, fresh):
        g.close()


def test_noalloc_refuses_a_wave_that_does_not_fit():
    """27 000 one-element layers with 32 workers: the records alone (64 bytes +
    32 pointers each) pass the 8 MiB of the static array.  PS_ERR_CAPACITY,
    nothing launched, nothing consumed; ps_aggregate takes the same wave."""
    from paper_2204_03211_amd import ParameterService
    layers = [1] * 27_000
    arena = torch.zeros(ParameterService.job_arena_bytes(layers) + 256, dtype=torch.uint8, device="cuda:0")
    svc = ParameterService(arena)
    job, nb = svc.register_job(layers, 32, 0.1, 0.9, 0.0)
    assert nb == 27_000
    g = torch.ones(svc.job_flat_numel(job), dtype=torch.float32, device="cuda:0")
    for w in range(32):
        svc.push_flat(job, w, g)
    wave = svc.pack_wave([job])
    with pytest.raises(PsError) as ei:
        svc.aggregate_noalloc(wave)
    assert ei.value.name == "PS_ERR_CAPACITY" and "8388608" in str(ei.value)
    torch.cuda.synchronize()
    p, v = svc.pull_flat(job)
    assert not p.any() and not v.any()
    assert svc.job_block_info(job, 0).round == 0
    svc.aggregate(wave)                           # the pushes are still there
    torch.cuda.synchronize()
    assert svc.job_block_info(job, nb - 1).round == 1
    assert float(svc.pull(job, 5)[0]) == float(np.float32(-3.2))     # p = 0 - 0.1 * 32
    svc.close()


def test_noalloc_on_the_full_packed_wave():
    """The twelve-job wave at full size (1743 blocks, 219 631 tiles: 4.2 MB of the
    8 MiB array) through the entry point that allocates nothing, two rounds (the
    second reuses the tables in the array), against ps_aggregate on a twin
    service with the same seeded inputs: every parameter, momentum value and
    telemetry pair identical."""
    specs = wl.packed_wave_jobs(42)
    ref, alt = GpuService(specs, 42), GpuService(specs, 42)
    wave_r, wave_a = ref.wave(), alt.wave()
    assert wave_r.tolist() == wave_a.tolist() and len(wave_r) == 1743
    for r in range(2):
        for g in (ref, alt):
            g.fill_grads(r)
            g.push_all()
        ref.svc.aggregate(wave_r)
        alt.svc.aggregate_noalloc(wave_a)
    assert_same(ref, alt, "full packed wave")
    ref.close(); alt.close()
