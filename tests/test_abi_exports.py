"""The shared library loads without a GPU and exports every function that
include/ps.h declares (no compute is called here)."""
import ctypes
import os
import re

from paper_2204_03211_amd import build, load_library
from paper_2204_03211_amd.binding import EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="ps.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ps_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 25
    lib = ctypes.CDLL(build.LIB) if os.path.exists(build.LIB) else load_library()
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(EXPORTS) == names        # the binding covers the same set


def test_version_and_strerror_without_device():
    L = load_library()
    assert L.ps_version() >= 100
    assert L.ps_strerror(0).decode() == "ok"
    assert L.ps_strerror(-999).decode() == "unknown status"


def test_scheduler_symbols_are_exported():
    from paper_2204_03211_amd.sched_binding import SCHED_EXPORTS
    names = declared_functions("ps_sched.h")
    assert len(names) == 24
    lib = load_library()
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(SCHED_EXPORTS) == names
