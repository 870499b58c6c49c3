"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], env=e,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    for r in (run("--gpus", "2"), run(env={"WORLD_SIZE": "4"})):
        assert r.returncode != 0
        assert b"one GPU" in r.stderr and r.stdout.strip() == b""


def test_traffic_figures_cover_the_timed_workloads():
    sys.path.insert(0, ROOT)
    import bench
    assert set(bench.MEASURED_TRAFFIC_PER_LAUNCH) == {"packed_wave", "vgg16", "resnet50", "alexnet"}
    assert bench.HBM_PEAK_GBS == 8000.0
    specs, seed = bench.specs_for("packed_wave")
    assert seed == 42 and len(specs) == 12 and [s.W for s in specs] == [16, 4, 2, 4, 8, 8, 4, 4, 4, 2, 8, 4]
