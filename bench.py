#!/usr/bin/env python3
"""Benchmark of the aggregation hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: pack
the wave, push every worker's gradient of every job, aggregate the wave (sum +
momentum-SGD update + telemetry, large- and small-block kernels), pull.
Inputs (gradients, parameters, momentum) are resident in HBM before the timed
region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Workloads: packed_wave (12 concurrent jobs, W in {2,4,8,16}; default), alexnet,
resnet50, vgg16, mlp.  --copy-calibration instead runs a plain 1 GiB device copy
a few times, so that profiler byte counters can be scaled by a kernel of known
traffic.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

# HBM bytes per ps_agg_wave launch from rocprofv3 FETCH_SIZE + WRITE_SIZE counters
# (each scaled by what the same counter reads for a 1 GiB copy), for the default
# configuration of a workload, as recorded under profiles/.  Each entry names the
# kernel sources it was measured with (kernel_hash()); with other sources the
# figure says nothing about the loaded kernel and the line reports null.
MEASURED_TRAFFIC = {
    "kernel_hash": "455f0af7709df7ad",
    "per_launch": {"packed_wave": 33.9590e9 / 110, "vgg16": 6.6483e9 / 17,
                   "resnet50": 2.0463e9 / 4, "alexnet": 2.9360e9 / 8},
}


def kernel_hash() -> str:
    """Hash of the files that define the kernels and their launch shape."""
    import hashlib
    h = hashlib.sha256()
    for f in ("ps_kernels.hip", "ps_internal.h"):
        with open(os.path.join(ROOT, "paper_2204_03211_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, default_config: bool, current_hash=None):
    """Counter traffic per launch for the roofline object, or None when it was
    not measured for this workload, this configuration or these kernel sources."""
    if not default_config:
        return None
    if (current_hash or kernel_hash()) != MEASURED_TRAFFIC["kernel_hash"]:
        return None
    return MEASURED_TRAFFIC["per_launch"].get(workload)


def specs_for(name: str):
    import workloads as wl
    if name == "packed_wave":
        return wl.packed_wave_jobs(42), 42
    return [wl.job_config(name)], 0


def cpu_baseline(gpu, wave_refs, budget_params: float = 6e9):
    """Time the oracle (one thread, as it stands) on a bounded sample of the same
    wave: every k-th block of the list, k chosen so the sample holds about
    budget_params worker-gradient elements.  Returns the JSON object."""
    import numpy as np
    import oracle
    import torch

    job_index = {j: i for i, j in enumerate(gpu.jobs)}
    sizes = []
    for j, b in wave_refs:
        ji = job_index[j]
        sizes.append(gpu.blocks[ji][b][2] * gpu.specs[ji].W)
    total = float(sum(sizes))
    k = max(1, int(round(total / budget_params)))
    sample = wave_refs[::k]
    work = []
    for j, b in sample:
        ji = job_index[j]
        s = gpu.specs[ji]
        layer, off, n, flat = gpu.blocks[ji][b]
        gs = [gpu.grads[ji][w][flat:flat + n].cpu().numpy() for w in range(s.W)]
        p = np.full(n, 0.01, dtype=np.float32)
        v = np.zeros(n, dtype=np.float32)
        work.append((gs, p, v, s))
    oracle.lib()
    t0 = time.perf_counter()
    for gs, p, v, s in work:
        oracle.aggregate_block(gs, p, v, s.lr, s.momentum, s.wd)
    dt = time.perf_counter() - t0
    n_params = sum(w[1].size for w in work)
    n_bytes = sum((4 * w[3].W + 16) * w[1].size for w in work)
    # second row: the same oracle function over the same blocks, one block per
    # call, from a pool of threads (blocks are independent; ctypes drops the GIL)
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(threads) as pool:
        t0 = time.perf_counter()
        list(pool.map(lambda w: oracle.aggregate_block(w[0], w[1], w[2], w[3].lr, w[3].momentum,
                                                       w[3].wd), work))
        dt_all = time.perf_counter() - t0
    return {
        "all_cores": {"value": n_params / dt_all, "unit": "params/s", "cores": threads,
                      "GB_per_s": n_bytes / dt_all / 1e9, "seconds": dt_all,
                      "note": "same oracle calls issued from a thread pool, one block per call"},
        "value": n_params / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
        "GB_per_s": n_bytes / dt / 1e9, "seconds": dt,
        "sample": (f"every block of the wave list" if k == 1 else f"every {k}-th block of the wave list")
                  + f": {len(work)} of {len(wave_refs)} blocks, {n_params} params, "
                    "single-threaded C++ oracle on host memory",
        "host_cpu": _cpu_model(), "host_cores_total": os.cpu_count(),
    }


def migration_bench(spec, reps: int, batched_only: bool = False, hold: int = 0, stagger: int = 0):
    """Move all blocks of one job from one context to another and back, reps
    times; the time is what a job would wait if nothing hid it (GPU time of the
    announce + copy calls, HIP events on the copy stream)."""
    import torch
    from paper_2204_03211_amd import ParameterService
    dev = torch.device("cuda:0")
    need = ParameterService.job_arena_bytes(spec.layer_numel) + 256
    arenas = [torch.zeros(need, dtype=torch.uint8, device=dev) for _ in range(2)]
    svcs = [ParameterService(a, store_hold_permille=hold, store_stagger_permille=stagger) for a in arenas]
    ja, nb = svcs[0].register_job(spec.layer_numel, spec.W, spec.lr, spec.momentum, spec.wd)
    jb, _ = svcs[1].register_shadow_job(spec.layer_numel, spec.W, spec.lr, spec.momentum, spec.wd)
    jobs = [ja, jb]
    torch.cuda.synchronize()
    times, host = [], []
    src = 0
    for _ in range(0 if batched_only else max(reps, 2)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        a.record()
        for blk in range(nb):
            svcs[src].migrate_begin(jobs[src], blk)
            svcs[src].migrate_copy(jobs[src], blk, svcs[1 - src], jobs[1 - src])
        b.record()
        host.append((time.perf_counter() - t0) * 1e3)
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b))
        src = 1 - src
    times, host = times[1:] or [float("nan")], host[1:] or [float("nan")]
    n_bytes = 8 * spec.n_params
    ms = sum(times) / len(times)
    # the same move as one batched call
    many = []
    for _ in range(max(reps, 2)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        svcs[src].migrate_many(jobs[src], list(range(nb)), svcs[1 - src], jobs[1 - src])
        b.record()
        torch.cuda.synchronize()
        many.append(a.elapsed_time(b))
        src = 1 - src
    many_ms = sum(many[1:]) / len(many[1:])
    out = {"migration": True, "model": spec.model, "blocks": nb, "params": spec.n_params,
           "bytes_moved": n_bytes, "gpu_ms": ms, "host_call_ms": sum(host) / len(host),
           "GB_per_s": n_bytes / ms / 1e6,
           "batched_gpu_ms": many_ms, "batched_GB_per_s": n_bytes / many_ms / 1e6,
           "batched_hbm_traffic_GB_per_s": 2 * n_bytes / many_ms / 1e6,
           "note": "bytes_moved = 8 bytes per parameter (parameters and momentum); each is read once and "
                   "written once, so HBM traffic is twice that; times are event times around the host "
                   "calls, launch latency included"}
    for s in svcs:
        s.close()
    return out


def _cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _per_wave_agg_ms(svc, step, n: int) -> dict:
    """ps_agg_wave's GPU time of n further waves, one reading per wave (the
    library reports sums, so each wave is the difference of two readings)."""
    svc.timing_enable(2)                          # every phase: four events a wave
    seen, each = 0.0, []
    for _ in range(n):
        step()
        tm = svc.timing_read()
        each.append(tm.agg_ms - seen)
        seen = tm.agg_ms
    svc.timing_enable(0)
    each.sort()
    return {"waves": n, "min": each[0], "median": each[len(each) // 2], "max": each[-1],
            "phases_mean": {"upload": tm.upload_ms / n, "ps_agg_wave": tm.agg_ms / n,
                            "ps_block_norms": tm.norms_ms / n, "gpu_total": tm.total_ms / n}}


def _path_split(svc, gpu, specs, n: int) -> dict:
    """Waves holding only the small-path blocks, and only the others, of the
    same jobs: ps_agg_wave's GPU time of each, per wave (median of n)."""
    from paper_2204_03211_amd.binding import WaveList

    refs = {"small": [], "large": []}
    grad_of = {}
    for ji, j in enumerate(gpu.jobs):
        for b in range(svc.job_n_blocks(j)):
            info = svc.job_block_info(j, b)
            refs["small" if info.small_path else "large"].append((j, b))
            grad_of[(j, b)] = [g.data_ptr() + 4 * info.flat_offset for g in gpu.grads[ji]]
    out = {}
    for name, lst in refs.items():
        if not lst:
            out[name] = {"only_ms_per_wave": None}
            continue
        wave = WaveList(lst)
        each = []
        for i in range(n + 1):
            for (j, b) in lst:
                for w, ptr in enumerate(grad_of[(j, b)]):
                    svc.push(j, b, w, ptr)
            if i == 1:
                svc.timing_enable(1)          # the first wave builds the plan: not read
            svc.aggregate(wave)
            if i >= 1:
                t = svc.timing_read().agg_ms
                each.append(t - sum(each))
        svc.timing_enable(0)
        each.sort()
        out[name] = {"only_ms_per_wave": each[len(each) // 2]}
    return out


def measure(workload: str, args, keep: bool):
    """Time args.steps steps of one workload; returns (json object, service, last wave)."""
    import torch
    from harness import GpuService

    specs, seed = specs_for(workload)
    t_setup = time.perf_counter()
    gpu = GpuService(specs, seed, small_block_elems=args.small_elems, launch_tiles=args.launch_tiles,
                     store_hold_permille=args.hold_permille, store_stagger_permille=args.stagger_permille)
    gpu.fill_grads(0)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    svc = gpu.svc

    def step():
        wave = svc.pack_wave(gpu.jobs)                       # a3
        for ji, s in enumerate(specs):                       # a2
            for w in range(s.W):
                svc.push_flat(gpu.jobs[ji], w, gpu.grads[ji][w])
        svc.aggregate(wave)                                  # a4-a7
        for j in gpu.jobs:                                   # a8
            svc.pull_flat(j)
        return wave

    for _ in range(args.warmup):
        wave = step()
    torch.cuda.synchronize()
    for ji, s in enumerate(specs):
        for w in range(s.W):
            svc.push_flat(gpu.jobs[ji], w, gpu.grads[ji][w])
    stats = svc.plan_wave(svc.pack_wave(gpu.jobs))
    svc.aggregate(svc.pack_wave(gpu.jobs))                   # consume the pushes again
    torch.cuda.synchronize()

    # the timed region: no library event on the stream, two events around all of it
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        wave = step()
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    region_ms = ev0.elapsed_time(ev1)
    # the same steps again, now with two library events a wave on the wave's stream (before the
    # first and after the last ps_agg_wave launch): the kernel's own time, for the roofline
    svc.timing_enable(1)
    for _ in range(args.steps):
        step()
    tm = svc.timing_read()
    svc.timing_enable(0)

    # outside the timed region: the same step once more, read wave by wave
    if args.no_side_configs:
        per_wave, paths = None, {"small": {}, "large": {}}
    else:
        per_wave = _per_wave_agg_ms(svc, step, args.steps)
        paths = _path_split(svc, gpu, specs, min(args.steps, 10))

    n_params = stats.n_params
    ms_per_step = dt / args.steps * 1e3
    value = n_params * args.steps / dt
    # the dominant kernel is ps_agg_wave; one wave is cut into several launches of it
    launches = max(tm.n_launches, 1)
    agg_ms_wave = tm.agg_ms / max(tm.n_waves, 1)
    bytes_per_launch = stats.algorithmic_bytes * tm.n_waves / launches
    avg_launch_ms = tm.agg_ms / launches
    achieved = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9 if avg_launch_ms > 0 else 0.0
    rates = svc.rates()
    out = {
        "metric": "aggregated params/sec and achieved HBM GB/s (% of MI355X peak), 1 GPU",
        "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": workload, "jobs": len(specs), "W": [s.W for s in specs],
            "job_shapes": [s.model for s in specs], "blocks": stats.n_blocks, "params": n_params,
            "block_cap_bytes": 4 << 20, "seed": seed,
            "algorithmic_bytes_per_step": stats.algorithmic_bytes,
        },
        "step_GB_per_s": stats.algorithmic_bytes * args.steps / dt / 1e9,
        "step_frac_of_hbm_peak": stats.algorithmic_bytes * args.steps / dt / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm", "kernel": "ps_agg_wave", "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(workload, not (args.small_elems or args.launch_tiles or args.hold_permille
                                                       or args.stagger_permille)),
            "kernel_hash": kernel_hash(),
            "algorithmic_bytes_per_launch": bytes_per_launch, "avg_launch_ms": avg_launch_ms,
            "launches": tm.n_launches, "launches_per_wave": stats.n_launches,
            "note": "avg_launch_ms = HIP-event time from the first to the last ps_agg_wave launch of a "
                    "wave (events on the wave's stream) divided by the launches in it, gaps between "
                    "launches included, over --steps waves that follow the timed region at once; the "
                    "timed region itself carries no library event, only one event at either end "
                    "(timed_region_event_ms: every kernel of the path)",
            "timed_region_event_ms": region_ms,
            "timed_region_GB_per_s": stats.algorithmic_bytes * args.steps / (region_ms * 1e-3) / 1e9,
        },
        "ps_agg_wave_ms_per_wave_timed": agg_ms_wave,
        "ps_agg_wave_ms_per_wave": per_wave,
        "small_path": {"blocks": stats.n_small_blocks, "bins": stats.n_small_bins,
                       "params": stats.small_params,
                       "algorithmic_bytes": stats.small_algorithmic_bytes, **paths["small"]},
        "large_path": {"blocks": stats.n_blocks - stats.n_small_blocks, "tiles": stats.n_large_tiles,
                       "params": stats.n_params - stats.small_params,
                       "algorithmic_bytes": stats.algorithmic_bytes - stats.small_algorithmic_bytes,
                       **paths["large"]},
        "setup_seconds": t_setup,
        "rates": {"read_TB_per_s": rates.read_bytes_per_sec / 1e12, "write_TB_per_s": rates.write_bytes_per_sec / 1e12,
                  "note": "what the library times launch phases with (built in, fitted on MI355X)"},
    }
    if not keep:
        gpu.close()
        del gpu
        torch.cuda.empty_cache()
        return out, None, None
    return out, gpu, wave


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="packed_wave")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-configs", action="store_true",
                    help="only the timed steps: skip the wave-by-wave and per-path passes and the "
                         "short single-job runs appended to the packed-wave line")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--kernel-hash", action="store_true",
                    help="print the hash of the kernel sources (what a traffic figure must name) and exit")
    ap.add_argument("--migration", action="store_true",
                    help="instead: time moving every block of --workload's first job to a second context")
    ap.add_argument("--migration-batched", action="store_true",
                    help="with --migration: only the one-call move of the whole job (for kernel profiles)")
    ap.add_argument("--path-split-only", action="store_true",
                    help="instead: only waves holding the small-path blocks alone, then the large-path blocks "
                         "alone, --steps of each (for kernel profiles of the two paths)")
    ap.add_argument("--small-elems", type=int, default=0, help="small-path threshold (0 = library default)")
    ap.add_argument("--launch-tiles", type=int, default=0, help="tiles per launch (0 = library default)")
    ap.add_argument("--hold-permille", type=int, default=0, help="store hold (0 = library default, <0 off)")
    ap.add_argument("--stagger-permille", type=int, default=0,
                    help="spread of a launch's store release (0 = library default, <0 all at once)")
    args = ap.parse_args()
    if args.kernel_hash:
        print(kernel_hash())
        return 0
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the service runs on one GPU; every block of every job lives on that GPU "
              "and no multi-GPU path exists; run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)              # an elementwise kernel: 1 read, 1 write
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "launches": 5}))
        return 0
    specs, seed = specs_for(args.workload)
    if args.migration:
        print(json.dumps(migration_bench(specs[0], args.steps, args.migration_batched, args.hold_permille,
                                         args.stagger_permille)))
        return 0
    if args.path_split_only:
        from harness import GpuService
        gpu = GpuService(specs, seed, small_block_elems=args.small_elems)
        gpu.fill_grads(0)
        torch.cuda.synchronize()
        gpu.push_all()
        st = gpu.svc.plan_wave(gpu.wave())
        gpu.svc.aggregate(gpu.wave())
        res = _path_split(gpu.svc, gpu, specs, args.steps)
        print(json.dumps({"path_split": True, "workload": args.workload, "waves_each": args.steps,
                          "small_path": {"blocks": st.n_small_blocks, "bins": st.n_small_bins,
                                         "params": st.small_params,
                                         "algorithmic_bytes": st.small_algorithmic_bytes, **res["small"]},
                          "large_path": {"blocks": st.n_blocks - st.n_small_blocks, "tiles": st.n_large_tiles,
                                         "algorithmic_bytes": st.algorithmic_bytes - st.small_algorithmic_bytes,
                                         **res["large"]}}))
        gpu.close()
        return 0
    out, gpu, wave = measure(args.workload, args, keep=True)
    if args.workload == "packed_wave" and not args.no_side_configs:
        # the single-job configurations, same step, fewer words: context for the headline line
        side = {}
        for name in ("alexnet", "resnet50", "vgg16"):
            o, _, _ = measure(name, args, keep=False)
            side[name] = {"params": o["config"]["params"], "W": o["config"]["W"][0],
                          "ms_per_step": o["ms_per_step"], "params_per_s": o["value"],
                          "step_GB_per_s": o["step_GB_per_s"],
                          "kernel_GB_per_s": o["roofline"]["achieved"],
                          "kernel_frac_of_hbm_peak": o["roofline"]["frac"]}
        out["single_job_configs"] = side
    if not args.no_cpu_baseline:
        try:
            out["cpu_baseline"] = cpu_baseline(gpu, wave.tolist())
        except (MemoryError, OSError, RuntimeError) as exc:   # the GPU figures stand without it
            out["cpu_baseline"] = {"value": None, "unit": "params/s", "cores": 1, "kind": "oracle",
                                   "sample": "not measured", "error": repr(exc)}
    gpu.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
