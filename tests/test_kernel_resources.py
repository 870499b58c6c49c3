"""The launch shape assumes that eight workgroups of the aggregation kernel fit
on a CU (8 waves per SIMD: at most 64 VGPRs; at most 20 KiB of LDS; no scratch).
Register use depends on how the compiler schedules the grouped loads, so it is
checked here from the compiler's own resource report (CPU only: hipcc
cross-compiles)."""
import os
import re
import subprocess
import tempfile

from paper_2204_03211_amd import build as B


def resource_report():
    src = os.path.join(B.CSRC, "ps_kernels.hip")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [B.hipcc(), *B.HIPCC_FLAGS, "-x", "hip", "-I", os.path.join(B.ROOT, "include"),
               "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", os.path.join(tmp, "k.o")]
        text = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, check=True).stdout.decode()
    out, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+(VGPRs|ScratchSize \[bytes/lane\]|LDS Size \[bytes/block\]|"
                      r"Occupancy \[waves/SIMD\]): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).split(" ")[0]] = int(m.group(2))
    return out


def test_aggregation_kernel_fits_eight_workgroups_per_cu():
    rep = resource_report()
    seen = set()
    for name, use in rep.items():
        m = re.search(r"ps_agg_waveILi(\d+)ELb(\d)", name)
        if not m:
            continue
        W, contract = int(m.group(1)), int(m.group(2))
        assert use["ScratchSize"] == 0, (name, use)
        assert use["LDS"] <= 20 * 1024, (name, use)
        if W >= 2:                       # the instantiations the launch tables are tuned for
            assert use["VGPRs"] <= 64 and use["Occupancy"] == 8, (name, use)
        else:                            # run-time W and W = 1: one workgroup fewer per CU is accepted
            assert use["VGPRs"] <= 72, (name, use)
        seen.add((W, contract))
    assert seen == {(w, c) for w in (0, 1, 2, 4, 8, 16) for c in (0, 1)}
