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
    assert set(bench.MEASURED_TRAFFIC["per_launch"]) == {"packed_wave", "vgg16", "resnet50", "alexnet"}
    assert bench.HBM_PEAK_GBS == 8000.0
    specs, seed = bench.specs_for("packed_wave")
    assert seed == 42 and len(specs) == 12 and [s.W for s in specs] == [16, 4, 2, 4, 8, 8, 4, 4, 4, 2, 8, 4]


def test_traffic_figure_is_tied_to_the_kernel_sources():
    """roofline.traffic repeats a profiler reading only for the kernel sources it
    was taken with, the default configuration and a profiled workload."""
    import bench
    h = bench.MEASURED_TRAFFIC["kernel_hash"]
    per = bench.MEASURED_TRAFFIC["per_launch"]
    assert bench.measured_traffic("packed_wave", True, current_hash=h) == per["packed_wave"]
    assert bench.measured_traffic("packed_wave", True, current_hash=h + "x") is None
    assert bench.measured_traffic("packed_wave", False, current_hash=h) is None
    assert bench.measured_traffic("mlp", True, current_hash=h) is None
    assert len(bench.kernel_hash()) == 16
    # against the files as they are now: either the recorded hash is current, or the line says null
    want = per["packed_wave"] if bench.kernel_hash() == h else None
    assert bench.measured_traffic("packed_wave", True) == want


def test_a_library_built_from_other_sources_is_stale(tmp_path, monkeypatch):
    from paper_2204_03211_amd import build
    src = tmp_path / "k.hip"
    src.write_text("// one\n")
    lib, stamp = tmp_path / "lib.so", tmp_path / "lib.so.srchash"
    monkeypatch.setattr(build, "LIB", str(lib))
    monkeypatch.setattr(build, "STAMP", str(stamp))
    monkeypatch.setattr(build, "source_files", lambda: [str(src)])
    assert build.is_stale()                               # nothing built
    lib.write_bytes(b"")
    assert build.is_stale()                               # a library of unknown origin
    stamp.write_text(build.source_hash([str(src)]) + "\n")
    assert not build.is_stale()
    src.write_text("// two\n")
    assert build.is_stale()                               # the source moved on, whatever the file times say
