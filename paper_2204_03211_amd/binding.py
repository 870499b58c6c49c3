"""ctypes binding of libps_agg.so: one Python method per C entry point of
include/ps.h, same names without the ps_ prefix.  Argument marshalling only:
every step of the aggregation path runs inside the library and its kernels.
PyTorch supplies device memory and streams.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

from . import build as _build

PS_MAX_W = 32
PS_OK = 0
FLAG_FP_CONTRACT = 1

ERRORS = {
    -1: "PS_ERR_ARG", -2: "PS_ERR_BAD_JOB", -3: "PS_ERR_BAD_BLOCK", -4: "PS_ERR_BAD_WORKER",
    -5: "PS_ERR_DUP_PUSH", -6: "PS_ERR_NOT_READY", -7: "PS_ERR_DUP_BLOCK", -8: "PS_ERR_ALIGN",
    -9: "PS_ERR_NOMEM", -10: "PS_ERR_NO_DEVICE", -11: "PS_ERR_HIP", -12: "PS_ERR_CAPACITY",
    -13: "PS_ERR_NOT_OWNER", -14: "PS_ERR_BUSY", -15: "PS_ERR_NO_ROOM",
}
OWNER_HERE, OWNER_LEAVING, OWNER_ELSEWHERE = 0, 1, 2


class PsError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{ERRORS.get(status, status)}: {text}")
        self.status = status
        self.name = ERRORS.get(status, str(status))


class Config(C.Structure):
    _fields_ = [("max_block_bytes", C.c_uint64), ("small_block_elems", C.c_uint32),
                ("flags", C.c_uint32), ("arena_dev", C.c_void_p), ("arena_bytes", C.c_uint64),
                ("launch_tiles", C.c_uint32), ("store_hold_permille", C.c_int32),
                ("store_stagger_permille", C.c_int32), ("reserved_", C.c_int32)]


class BlockRef(C.Structure):
    _fields_ = [("job", C.c_int32), ("block", C.c_int32)]


class BlockInfo(C.Structure):
    _fields_ = [("layer", C.c_int32), ("W", C.c_int32), ("layer_offset", C.c_int64),
                ("numel", C.c_int64), ("flat_offset", C.c_int64), ("round", C.c_int64),
                ("push_mask", C.c_uint32), ("small_path", C.c_uint32), ("owner", C.c_uint32),
                ("reserved_", C.c_uint32)]


class BlockStats(C.Structure):
    _fields_ = [("grad_norm2", C.c_double), ("round", C.c_int64)]


class WaveStats(C.Structure):
    _fields_ = [("n_blocks", C.c_int64), ("n_params", C.c_int64), ("n_large_tiles", C.c_int64),
                ("n_small_blocks", C.c_int64), ("n_small_bins", C.c_int64),
                ("small_params", C.c_int64), ("algorithmic_bytes", C.c_uint64),
                ("small_algorithmic_bytes", C.c_uint64), ("n_launches", C.c_int64),
                ("est_seconds", C.c_double)]


class Rates(C.Structure):
    _fields_ = [("read_bytes_per_sec", C.c_double), ("write_bytes_per_sec", C.c_double),
                ("reserved_", C.c_int32 * 2)]


class Timing(C.Structure):
    _fields_ = [("n_waves", C.c_int64), ("n_launches", C.c_int64), ("upload_ms", C.c_double),
                ("agg_ms", C.c_double), ("norms_ms", C.c_double), ("total_ms", C.c_double)]


EXPORTS = [
    "ps_create", "ps_destroy", "ps_job_arena_bytes", "ps_register_job", "ps_register_shadow_job",
    "ps_unregister_job", "ps_split_ready", "ps_migrate_begin", "ps_migrate_cancel", "ps_migrate_copy",
    "ps_migrate_many", "ps_estimate_wave",
    "ps_job_n_blocks", "ps_job_flat_numel", "ps_job_block_info", "ps_push", "ps_push_flat",
    "ps_pack_wave", "ps_plan_wave", "ps_aggregate", "ps_aggregate_noalloc", "ps_pull", "ps_pull_momentum", "ps_pull_flat", "ps_pull_copy",
    "ps_telemetry", "ps_rates", "ps_timing_enable", "ps_timing_read", "ps_strerror", "ps_last_error", "ps_version",
]

_lib = None


def load_library() -> C.CDLL:
    """Load the in-tree library; build it first if there is none or if it was
    not built from the present sources (an edited kernel must never be tested
    through an old binary).  There is no fallback: without the library, or
    without a compiler to refresh a stale one, this raises."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        _build.build()
    L = C.CDLL(_build.LIB)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    P = C.POINTER
    L.ps_create.argtypes = [P(Config), P(vp)]
    L.ps_destroy.argtypes = [vp]
    L.ps_destroy.restype = None
    L.ps_job_arena_bytes.argtypes = [P(Config), P(i64), i32, P(u64)]
    L.ps_register_job.argtypes = [vp, P(i64), i32, i32, C.c_float, C.c_float, C.c_float,
                                  P(vp), vp, P(i32), P(i32)]
    L.ps_register_shadow_job.argtypes = [vp, P(i64), i32, i32, C.c_float, C.c_float, C.c_float,
                                         vp, P(i32), P(i32)]
    L.ps_split_ready.argtypes = [vp, P(BlockRef), i64, P(BlockRef), P(i64), P(BlockRef), P(i64)]
    L.ps_migrate_begin.argtypes = [vp, i32, i32]
    L.ps_migrate_cancel.argtypes = [vp, i32, i32]
    L.ps_migrate_copy.argtypes = [vp, i32, i32, vp, i32, vp]
    L.ps_migrate_many.argtypes = [vp, i32, C.POINTER(i32), i32, vp, i32, vp]
    L.ps_unregister_job.argtypes = [vp, i32]
    L.ps_job_n_blocks.argtypes = [vp, i32]
    L.ps_job_flat_numel.argtypes = [vp, i32]
    L.ps_job_flat_numel.restype = i64
    L.ps_job_block_info.argtypes = [vp, i32, i32, P(BlockInfo)]
    L.ps_push.argtypes = [vp, i32, i32, i32, vp]
    L.ps_push_flat.argtypes = [vp, i32, i32, vp]
    L.ps_pack_wave.argtypes = [vp, P(i32), i32, P(BlockRef), i64, P(i64)]
    L.ps_plan_wave.argtypes = [vp, P(BlockRef), i64, P(WaveStats)]
    L.ps_estimate_wave.argtypes = [vp, P(BlockRef), i64, P(WaveStats)]
    L.ps_aggregate.argtypes = [vp, P(BlockRef), i64, vp]
    L.ps_aggregate_noalloc.argtypes = [vp, P(BlockRef), i64, vp]
    L.ps_pull.argtypes = [vp, i32, i32, P(vp), P(i64)]
    L.ps_pull_momentum.argtypes = [vp, i32, i32, P(vp), P(i64)]
    L.ps_pull_flat.argtypes = [vp, i32, P(vp), P(vp), P(i64)]
    L.ps_pull_copy.argtypes = [vp, i32, i32, vp, vp]
    L.ps_telemetry.argtypes = [vp, i32, i32, P(BlockStats)]
    L.ps_rates.argtypes = [vp, P(Rates)]
    L.ps_timing_enable.argtypes = [vp, i32]
    L.ps_timing_read.argtypes = [vp, P(Timing)]
    L.ps_strerror.argtypes = [i32]
    L.ps_strerror.restype = C.c_char_p
    L.ps_last_error.argtypes = [vp]
    L.ps_last_error.restype = C.c_char_p
    L.ps_version.argtypes = []
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int:   # default: make the status type explicit
            fn.restype = i32
    _lib = L
    return L


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


class WaveList:
    """A host array of (job, block) references, kept in C layout."""

    def __init__(self, refs: Sequence[Tuple[int, int]] = (), _arr=None, _n: int = 0):
        if _arr is not None:
            self.arr, self.n = _arr, _n
        else:
            self.n = len(refs)
            self.arr = (BlockRef * max(self.n, 1))()
            for i, (j, b) in enumerate(refs):
                self.arr[i].job, self.arr[i].block = j, b

    def __len__(self) -> int:
        return self.n

    def tolist(self) -> List[Tuple[int, int]]:
        return [(self.arr[i].job, self.arr[i].block) for i in range(self.n)]


class ParameterService:
    """Thin owner of a ps_ctx.  arena: a 1-D torch.uint8/float32 CUDA tensor the
    service carves master copies from (None = planning context, no device)."""

    def __init__(self, arena: Optional[torch.Tensor] = None, max_block_bytes: int = 0,
                 small_block_elems: int = 0, flags: int = 0, launch_tiles: int = 0,
                 store_hold_permille: int = 0, store_stagger_permille: int = 0):
        self.L = load_library()
        self.arena = arena
        cfg = Config(max_block_bytes, small_block_elems, flags,
                     arena.data_ptr() if arena is not None else None,
                     arena.numel() * arena.element_size() if arena is not None else 0,
                     launch_tiles, store_hold_permille, store_stagger_permille, 0)
        self.cfg = cfg
        self.ctx = C.c_void_p()
        self._check(self.L.ps_create(C.byref(cfg), C.byref(self.ctx)))

    # -- helpers -------------------------------------------------------------
    def _check(self, status: int) -> int:
        if status < 0:
            text = self.L.ps_strerror(status).decode()
            if status in (-11, -12) and self.ctx:
                text += " (" + self.L.ps_last_error(self.ctx).decode() + ")"
            raise PsError(status, text)
        return status

    @staticmethod
    def job_arena_bytes(layer_numel: Sequence[int], max_block_bytes: int = 0) -> int:
        L = load_library()
        cfg = Config(max_block_bytes, 0, 0, None, 0, 0, 0)
        arr = (C.c_int64 * len(layer_numel))(*layer_numel)
        out = C.c_uint64()
        st = L.ps_job_arena_bytes(C.byref(cfg), arr, len(layer_numel), C.byref(out))
        if st < 0:
            raise PsError(st, L.ps_strerror(st).decode())
        return out.value

    def close(self) -> None:
        if self.ctx:
            self.L.ps_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C entry points ----------------------------------------------------
    def register_job(self, layer_numel: Sequence[int], W: int, lr: float, momentum: float,
                     wd: float, init_params: Optional[Sequence[Optional[torch.Tensor]]] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> Tuple[int, int]:
        n = len(layer_numel)
        arr = (C.c_int64 * max(n, 1))(*layer_numel)
        ptrs = None
        if init_params is not None:
            assert len(init_params) == n
            for t, ne in zip(init_params, layer_numel):
                assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
                                     and t.numel() == ne)
            ptrs = (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in init_params])
        job, nb = C.c_int32(), C.c_int32()
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_register_job(self.ctx, arr, n, W, lr, momentum, wd, ptrs, sp,
                                           C.byref(job), C.byref(nb)))
        return job.value, nb.value

    def register_shadow_job(self, layer_numel: Sequence[int], W: int, lr: float, momentum: float,
                            wd: float, stream: Optional[torch.cuda.Stream] = None) -> Tuple[int, int]:
        n = len(layer_numel)
        arr = (C.c_int64 * max(n, 1))(*layer_numel)
        job, nb = C.c_int32(), C.c_int32()
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_register_shadow_job(self.ctx, arr, n, W, lr, momentum, wd, sp,
                                                  C.byref(job), C.byref(nb)))
        return job.value, nb.value

    def split_ready(self, wave: WaveList) -> Tuple[WaveList, WaveList]:
        ready = (BlockRef * max(wave.n, 1))()
        late = (BlockRef * max(wave.n, 1))()
        nr, nl = C.c_int64(), C.c_int64()
        self._check(self.L.ps_split_ready(self.ctx, wave.arr, wave.n, ready, C.byref(nr), late, C.byref(nl)))
        return WaveList(_arr=ready, _n=nr.value), WaveList(_arr=late, _n=nl.value)

    def migrate_begin(self, job: int, block: int) -> None:
        self._check(self.L.ps_migrate_begin(self.ctx, job, block))

    def migrate_cancel(self, job: int, block: int) -> None:
        self._check(self.L.ps_migrate_cancel(self.ctx, job, block))

    def migrate_copy(self, job: int, block: int, dst: "ParameterService", dst_job: int,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_migrate_copy(self.ctx, job, block, dst.ctx, dst_job, sp))

    def migrate_many(self, job: int, blocks: Sequence[int], dst: "ParameterService", dst_job: int,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
        arr = (C.c_int32 * max(len(blocks), 1))(*blocks)
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_migrate_many(self.ctx, job, arr, len(blocks), dst.ctx, dst_job, sp))

    def unregister_job(self, job: int) -> None:
        self._check(self.L.ps_unregister_job(self.ctx, job))

    def job_n_blocks(self, job: int) -> int:
        return self._check(self.L.ps_job_n_blocks(self.ctx, job))

    def job_flat_numel(self, job: int) -> int:
        v = self.L.ps_job_flat_numel(self.ctx, job)
        if v < 0:
            self._check(int(v))
        return int(v)

    def job_block_info(self, job: int, block: int) -> BlockInfo:
        out = BlockInfo()
        self._check(self.L.ps_job_block_info(self.ctx, job, block, C.byref(out)))
        return out

    def push(self, job: int, block: int, worker: int, grad) -> None:
        """grad: a CUDA float32 tensor or a raw device address."""
        ptr = grad.data_ptr() if isinstance(grad, torch.Tensor) else int(grad)
        self._check(self.L.ps_push(self.ctx, job, block, worker, ptr))

    def push_flat(self, job: int, worker: int, grad_flat) -> None:
        ptr = grad_flat.data_ptr() if isinstance(grad_flat, torch.Tensor) else int(grad_flat)
        self._check(self.L.ps_push_flat(self.ctx, job, worker, ptr))

    def pack_wave(self, jobs: Sequence[int]) -> WaveList:
        ja = (C.c_int32 * max(len(jobs), 1))(*jobs)
        need = C.c_int64()
        st = self.L.ps_pack_wave(self.ctx, ja, len(jobs), None, 0, C.byref(need))
        if st not in (0, -12):
            self._check(st)
        arr = (BlockRef * max(need.value, 1))()
        self._check(self.L.ps_pack_wave(self.ctx, ja, len(jobs), arr, need.value, C.byref(need)))
        return WaveList(_arr=arr, _n=need.value)

    def plan_wave(self, wave: WaveList) -> WaveStats:
        out = WaveStats()
        self._check(self.L.ps_plan_wave(self.ctx, wave.arr, wave.n, C.byref(out)))
        return out

    def estimate_wave(self, wave: WaveList) -> WaveStats:
        out = WaveStats()
        self._check(self.L.ps_estimate_wave(self.ctx, wave.arr, wave.n, C.byref(out)))
        return out

    def aggregate(self, wave: WaveList, stream: Optional[torch.cuda.Stream] = None) -> None:
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_aggregate(self.ctx, wave.arr, wave.n, sp))

    def aggregate_noalloc(self, wave: WaveList, stream: Optional[torch.cuda.Stream] = None) -> None:
        sp = _stream_ptr(stream) if self.arena is not None else None
        self._check(self.L.ps_aggregate_noalloc(self.ctx, wave.arr, wave.n, sp))

    def pull(self, job: int, block: int) -> torch.Tensor:
        """The block's parameters as a view into the arena (no copy)."""
        ptr, n = C.c_void_p(), C.c_int64()
        self._check(self.L.ps_pull(self.ctx, job, block, C.byref(ptr), C.byref(n)))
        return self._view(ptr.value, n.value)

    def pull_copy(self, job: int, block: int, dst: torch.Tensor,
                  stream: Optional[torch.cuda.Stream] = None) -> None:
        """Copy the block's parameters into dst (CUDA float32, at least numel elements)."""
        sp = _stream_ptr(stream) if self.arena is not None else None
        ptr = dst.data_ptr() if isinstance(dst, torch.Tensor) else int(dst)
        self._check(self.L.ps_pull_copy(self.ctx, job, block, ptr, sp))

    def pull_momentum(self, job: int, block: int) -> torch.Tensor:
        ptr, n = C.c_void_p(), C.c_int64()
        self._check(self.L.ps_pull_momentum(self.ctx, job, block, C.byref(ptr), C.byref(n)))
        return self._view(ptr.value, n.value)

    def pull_flat(self, job: int) -> Tuple[torch.Tensor, torch.Tensor]:
        p, v, n = C.c_void_p(), C.c_void_p(), C.c_int64()
        self._check(self.L.ps_pull_flat(self.ctx, job, C.byref(p), C.byref(v), C.byref(n)))
        return self._view(p.value, n.value), self._view(v.value, n.value)

    def telemetry(self, job: int, block: int) -> BlockStats:
        out = BlockStats()
        self._check(self.L.ps_telemetry(self.ctx, job, block, C.byref(out)))
        return out

    def rates(self) -> Rates:
        out = Rates()
        self._check(self.L.ps_rates(self.ctx, C.byref(out)))
        return out

    def timing_enable(self, on: bool) -> None:
        self._check(self.L.ps_timing_enable(self.ctx, int(on)))

    def timing_read(self) -> Timing:
        out = Timing()
        self._check(self.L.ps_timing_read(self.ctx, C.byref(out)))
        return out

    def version(self) -> int:
        return self.L.ps_version()

    # -- arena views -------------------------------------------------------------
    def _view(self, ptr: int, numel: int) -> torch.Tensor:
        base = self.arena.data_ptr()
        off = ptr - base
        assert 0 <= off and off + 4 * numel <= self.arena.numel() * self.arena.element_size()
        flat = self.arena.view(torch.uint8)[off:off + 4 * numel]
        return flat.view(torch.float32)
