"""CPU oracle for model aggregation -- TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  The product library never does, and this package never imports
the product library.  The arithmetic lives in ps_oracle.cpp (plain C++, one
thread, no fused multiply-add); this file compiles it with g++, binds it with
ctypes, and adds a small stateful model of a service (jobs, blocks, rounds) on
numpy arrays so a whole multi-job run can be replayed on the CPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ps_oracle.cpp")
_LIB = os.path.join(_HERE, "libps_oracle.so")

# no contraction, no value-changing optimisation, no vector-math rewrites of the
# summation order: -O2 keeps IEEE semantics as long as fast-math stays off.
CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]

BLOCK_CAP_ELEMS = 1 << 20  # "<= 4 MB" blocks read as 4 MiB = 2^20 binary32 values


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["g++", *CXXFLAGS, "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        fpp = C.POINTER(C.c_void_p)
        L.orc_split_layers.restype = C.c_int64
        L.orc_split_layers.argtypes = [i64p, C.c_int32, C.c_int64, i32p, i64p, i64p, C.c_int64]
        L.orc_arrival_order.restype = None
        L.orc_arrival_order.argtypes = [i32p, C.c_int32, i32p]
        L.orc_interleave.restype = None
        L.orc_interleave.argtypes = [i32p, C.c_int32, i32p, i32p]
        L.orc_aggregate_block.restype = None
        L.orc_aggregate_block.argtypes = [C.c_int32, C.c_int64, fpp, C.c_void_p, C.c_void_p,
                                          C.c_float, C.c_float, C.c_float, C.POINTER(C.c_double)]
        L.orc_sum_block.restype = None
        L.orc_sum_block.argtypes = [C.c_int32, C.c_int64, fpp, C.c_void_p]
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def split_layers(layer_numel: Sequence[int], cap_elems: int = BLOCK_CAP_ELEMS
                 ) -> List[Tuple[int, int, int]]:
    """[(layer, offset in layer, numel)] for every block, registration order."""
    n = len(layer_numel)
    ln = (C.c_int64 * max(n, 1))(*[int(x) for x in layer_numel])
    cap = sum(-(-int(x) // cap_elems) for x in layer_numel) if cap_elems > 0 else 0
    cap = max(cap, 1)
    ol, oo, on = (C.c_int32 * cap)(), (C.c_int64 * cap)(), (C.c_int64 * cap)()
    nb = lib().orc_split_layers(ln, n, cap_elems, ol, oo, on, cap)
    if nb < 0:
        raise ValueError("invalid split arguments")
    return [(ol[i], oo[i], on[i]) for i in range(nb)]


def arrival_order(block_layer: Sequence[int]) -> List[int]:
    n = len(block_layer)
    bl = (C.c_int32 * max(n, 1))(*block_layer)
    out = (C.c_int32 * max(n, 1))()
    lib().orc_arrival_order(bl, n, out)
    return list(out[:n])


def interleave(n_blocks_per_job: Sequence[int]) -> List[Tuple[int, int]]:
    """[(job index, position k in that job's arrival sequence)] of one wave."""
    nj = len(n_blocks_per_job)
    tot = int(sum(n_blocks_per_job))
    nb = (C.c_int32 * max(nj, 1))(*n_blocks_per_job)
    oj, ok = (C.c_int32 * max(tot, 1))(), (C.c_int32 * max(tot, 1))()
    lib().orc_interleave(nb, nj, oj, ok)
    return [(oj[i], ok[i]) for i in range(tot)]


def sum_block(grads: Sequence[np.ndarray]) -> np.ndarray:
    gs = [_f32(g) for g in grads]
    n = gs[0].size
    ptrs = (C.c_void_p * len(gs))(*[g.ctypes.data for g in gs])
    out = np.empty(n, dtype=np.float32)
    lib().orc_sum_block(len(gs), n, ptrs, out.ctypes.data)
    return out


def aggregate_block(grads: Sequence[np.ndarray], p: np.ndarray, v: np.ndarray,
                    lr: float, mu: float, wd: float) -> float:
    """Update p and v (float32, contiguous) in place; returns sum_i S[i]^2."""
    assert p.dtype == np.float32 and v.dtype == np.float32
    assert p.flags.c_contiguous and v.flags.c_contiguous and p.size == v.size
    gs = [_f32(g) for g in grads]
    assert all(g.size == p.size for g in gs) and len(gs) >= 1
    ptrs = (C.c_void_p * len(gs))(*[g.ctypes.data for g in gs])
    n2 = C.c_double(0.0)
    lib().orc_aggregate_block(len(gs), p.size, ptrs, p.ctypes.data, v.ctypes.data,
                              C.c_float(lr), C.c_float(mu), C.c_float(wd), C.byref(n2))
    return n2.value


# ---------------------------------------------------------------------------
# A stateful model of the service on numpy arrays
# ---------------------------------------------------------------------------
@dataclass
class OracleJob:
    layer_numel: Tuple[int, ...]
    W: int
    lr: float
    mu: float
    wd: float
    cap_elems: int = BLOCK_CAP_ELEMS
    blocks: List[Tuple[int, int, int]] = field(default_factory=list)
    p: List[np.ndarray] = field(default_factory=list)      # one array per layer
    v: List[np.ndarray] = field(default_factory=list)
    round: List[int] = field(default_factory=list)          # per block
    norm2: List[float] = field(default_factory=list)        # per block, last round

    def __post_init__(self):
        self.blocks = split_layers(self.layer_numel, self.cap_elems)
        self.p = [np.zeros(n, dtype=np.float32) for n in self.layer_numel]
        self.v = [np.zeros(n, dtype=np.float32) for n in self.layer_numel]
        self.round = [0] * len(self.blocks)
        self.norm2 = [0.0] * len(self.blocks)

    def arrival(self) -> List[int]:
        return arrival_order([b[0] for b in self.blocks])

    def block_view(self, arrs: List[np.ndarray], b: int) -> np.ndarray:
        layer, off, n = self.blocks[b]
        return arrs[layer][off:off + n]

    def aggregate(self, b: int, grads: Sequence[np.ndarray]) -> None:
        """grads: W arrays holding this block's gradient from workers 0..W-1."""
        assert len(grads) == self.W
        self.norm2[b] = aggregate_block(grads, self.block_view(self.p, b),
                                        self.block_view(self.v, b), self.lr, self.mu, self.wd)
        self.round[b] += 1


def pack_wave(jobs: Sequence[OracleJob]) -> List[Tuple[int, int]]:
    """[(job index, block id)] of one wave in which every job contributes one
    round: each job's blocks in arrival order, jobs interleaved by position."""
    orders = [j.arrival() for j in jobs]
    return [(j, orders[j][k]) for j, k in interleave([len(o) for o in orders])]
