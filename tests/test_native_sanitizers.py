"""Host code under AddressSanitizer + UBSan (CPU only): the service's planning
paths and the scheduler through a small C++ driver, and the oracle's C++ under
the same sanitizers through its own self-check; the service's locking under
ThreadSanitizer with several threads on two shared contexts."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2204_03211_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"),
                    reason="needs g++ and the HIP headers")
def test_service_and_scheduler_host_code_is_clean_under_asan_ubsan():
    with tempfile.TemporaryDirectory() as td:
        exe = os.path.join(td, "driver")
        cmd = ["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
               "-I", os.path.join(ROOT, "include"),
               os.path.join(ROOT, "tests", "native", "host_sanitize_driver.cpp"),
               os.path.join(CSRC, "ps_service.cpp"), os.path.join(CSRC, "ps_sched.cpp"),
               os.path.join(CSRC, "ps_pmaster.cpp"),
               "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread", "-o", exe]
        subprocess.check_call(cmd)
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")
        out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
        assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
        assert "host sanitize driver: ok" in out.stdout


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"),
                    reason="needs g++ and the HIP headers")
def test_service_locking_is_clean_under_tsan():
    """Four threads register, push, plan, estimate, inspect and unregister jobs of
    their own on two shared contexts and ask for migrations in both directions
    (two contexts locked per call, in address order): no data race, no lock-order
    inversion, every status as expected."""
    with tempfile.TemporaryDirectory() as td:
        exe = os.path.join(td, "driver_tsan")
        cmd = ["g++", "-std=c++17", "-fsanitize=thread", "-fno-omit-frame-pointer", "-g", "-O1",
               "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
               os.path.join(ROOT, "tests", "native", "host_sanitize_driver.cpp"),
               os.path.join(CSRC, "ps_service.cpp"), os.path.join(CSRC, "ps_sched.cpp"),
               os.path.join(CSRC, "ps_pmaster.cpp"),
               "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread", "-o", exe]
        subprocess.check_call(cmd)
        env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:second_deadlock_stack=1")
        out = subprocess.run([exe, "threads"], env=env, capture_output=True, text=True, timeout=300)
        assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
        assert "host thread driver: ok" in out.stdout
        assert "ThreadSanitizer" not in out.stderr


def test_oracle_cpp_is_clean_under_asan_ubsan():
    src = os.path.join(ROOT, "oracle", "ps_oracle.cpp")
    main = r"""
#include <cstdint>
#include <cstdio>
#include <vector>
extern "C" {
int64_t orc_split_layers(const int64_t*, int32_t, int64_t, int32_t*, int64_t*, int64_t*, int64_t);
void orc_arrival_order(const int32_t*, int32_t, int32_t*);
void orc_interleave(const int32_t*, int32_t, int32_t*, int32_t*);
void orc_aggregate_block(int32_t, int64_t, const float* const*, float*, float*, float, float, float, double*);
void orc_sum_block(int32_t, int64_t, const float* const*, float*);
}
int main() {
  std::vector<int64_t> layers = {1000, 37, 4099, 64, 1};
  std::vector<int32_t> bl(64); std::vector<int64_t> bo(64), bn(64);
  int64_t nb = orc_split_layers(layers.data(), 5, 1000, bl.data(), bo.data(), bn.data(), 64);
  if (nb != 1 + 1 + 5 + 1 + 1) return 1;
  std::vector<int32_t> order(nb);
  orc_arrival_order(bl.data(), (int32_t)nb, order.data());
  int32_t per[3] = {5, 0, 9};
  std::vector<int32_t> oj(14), ok(14);
  orc_interleave(per, 3, oj.data(), ok.data());
  const int W = 5; const int64_t n = 1237;
  std::vector<std::vector<float>> g(W, std::vector<float>(n, 0.25f));
  std::vector<const float*> gp; for (auto& v : g) gp.push_back(v.data());
  std::vector<float> p(n, 1.0f), v(n, 0.0f), s(n);
  double n2 = 0;
  for (int r = 0; r < 3; ++r) orc_aggregate_block(W, n, gp.data(), p.data(), v.data(), 0.1f, 0.9f, 1e-4f, &n2);
  orc_sum_block(W, n, gp.data(), s.data());
  if (s[0] != 1.25f || n2 != 1.25 * 1.25 * n) return 2;
  std::printf("oracle sanitize: ok\n");
  return 0;
}
"""
    with tempfile.TemporaryDirectory() as td:
        mp, exe = os.path.join(td, "main.cpp"), os.path.join(td, "o")
        open(mp, "w").write(main)
        subprocess.check_call(["g++", "-std=c++17", *SAN, "-ffp-contract=off", src, mp, "-o", exe])
        env = dict(os.environ, ASAN_OPTIONS="abort_on_error=1")
        out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
        assert out.returncode == 0, out.stdout + out.stderr[-3000:]
        assert "oracle sanitize: ok" in out.stdout
