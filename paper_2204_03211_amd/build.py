"""Compile the service library for gfx950 with hipcc, in-tree.

    python -m paper_2204_03211_amd.build        # (re)build libps_agg.so
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libps_agg.so")
SOURCES = ["ps_service.cpp", "ps_sched.cpp", "ps_pmaster.cpp", "ps_kernels.hip"]
HEADERS = [os.path.join(CSRC, "ps_internal.h"), os.path.join(ROOT, "include", "ps.h"),
           os.path.join(ROOT, "include", "ps_sched.h")]

# -ffp-contract=off: the update's multiplies and adds must stay separate
# roundings.  The packed-fp32 feature is switched off for device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


STAMP = LIB + ".srchash"


def source_files():
    return [os.path.join(CSRC, s) for s in SOURCES] + HEADERS


def source_hash(files=None) -> str:
    """Hash of everything the library is built from: sources, headers, flags.
    File times are not used: a copied tree has arbitrary ones."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for f in (files if files is not None else source_files()):
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:20]


def is_stale() -> bool:
    """True unless the built library was made from exactly the present sources
    (build() records their hash next to it)."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return True
    with open(STAMP) as fh:
        return fh.read().strip() != source_hash()


def build(verbose: bool = False) -> str:
    objs = []
    procs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc(), *HIPCC_FLAGS, "-x", "hip", "-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # the host pass does not know the device-only feature flag: harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + text)
        if verbose and text.strip():
            print(text)
    stamp = source_hash()          # of what was just compiled
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.check_call(cmd)
    with open(STAMP, "w") as fh:
        fh.write(stamp + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
