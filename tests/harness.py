"""Shared scaffolding of the GPU parity tests, the smoke check and the benchmark:
build a service on the GPU from job specs, fill seeded gradients, and replay
the same run on the CPU oracle.  Values come from workloads/ only; the oracle
side never sees anything the HIP path computed."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

import workloads as wl
from paper_2204_03211_amd import ParameterService, WaveList


def layer_values(seed: int, kind: str, ids: Tuple[int, ...], n: int, std: float,
                 device, start: int = 0) -> torch.Tensor:
    out = torch.empty(n, dtype=torch.float32, device=device)
    return wl.fill_normal_like(out, wl.stream_key(seed, kind, *ids), std, start=start)


class GpuService:
    """Jobs registered on the GPU with one flat gradient buffer per (job, worker)."""

    def __init__(self, specs: Sequence[wl.JobSpec], seed: int, max_block_bytes: int = 0,
                 small_block_elems: int = 0, flags: int = 0, device="cuda:0",
                 grad_pad_elems: int = 0, launch_tiles: int = 0, store_hold_permille: int = 0,
                 store_stagger_permille: int = 0):
        self.specs, self.seed, self.dev = list(specs), seed, torch.device(device)
        need = sum(ParameterService.job_arena_bytes(s.layer_numel, max_block_bytes) + 256 for s in specs)
        self.arena = torch.empty(need, dtype=torch.uint8, device=self.dev)
        self.svc = ParameterService(self.arena, max_block_bytes, small_block_elems, flags,
                                    launch_tiles, store_hold_permille, store_stagger_permille)
        self.jobs: List[int] = []
        self.layer_flat: List[List[int]] = []     # flat offset of each layer, per job
        self.blocks: List[List[Tuple[int, int, int, int]]] = []  # (layer, layer_off, numel, flat_off)
        self.grads: List[List[torch.Tensor]] = []
        for ji, s in enumerate(specs):
            init = [layer_values(seed, "param", (ji, l), n, s.param_std, self.dev)
                    for l, n in enumerate(s.layer_numel)]
            job, nb = self.svc.register_job(s.layer_numel, s.W, s.lr, s.momentum, s.wd, init)
            torch.cuda.synchronize()
            del init
            self.jobs.append(job)
            infos = [self.svc.job_block_info(job, b) for b in range(nb)]
            self.blocks.append([(i.layer, i.layer_offset, i.numel, i.flat_offset) for i in infos])
            lf = [0] * len(s.layer_numel)
            for i in infos:
                if i.layer_offset == 0:
                    lf[i.layer] = i.flat_offset
            self.layer_flat.append(lf)
            fn = self.svc.job_flat_numel(job)
            # distinct allocation per worker; an optional odd pad staggers their addresses
            self.grads.append([torch.zeros(fn + grad_pad_elems * (w + 1), dtype=torch.float32,
                                           device=self.dev)[grad_pad_elems * (w + 1):]
                               if grad_pad_elems else
                               torch.zeros(fn, dtype=torch.float32, device=self.dev)
                               for w in range(s.W)])

    def fill_grads(self, rnd: int) -> None:
        for ji, s in enumerate(self.specs):
            for w in range(s.W):
                g = self.grads[ji][w]
                for l, n in enumerate(s.layer_numel):
                    o = self.layer_flat[ji][l]
                    wl.fill_normal_like(g[o:o + n], wl.stream_key(self.seed, "grad", ji, w, rnd, l),
                                        s.grad_std)

    def push_all(self) -> None:
        for ji, s in enumerate(self.specs):
            for w in range(s.W):
                self.svc.push_flat(self.jobs[ji], w, self.grads[ji][w])

    def wave(self) -> WaveList:
        return self.svc.pack_wave(self.jobs)

    def step(self, wave: Optional[WaveList] = None) -> None:
        self.push_all()
        self.svc.aggregate(wave if wave is not None else self.wave())

    def layer_param(self, ji: int, l: int) -> torch.Tensor:
        p, _ = self.svc.pull_flat(self.jobs[ji])
        o = self.layer_flat[ji][l]
        return p[o:o + self.specs[ji].layer_numel[l]]

    def layer_momentum(self, ji: int, l: int) -> torch.Tensor:
        _, v = self.svc.pull_flat(self.jobs[ji])
        o = self.layer_flat[ji][l]
        return v[o:o + self.specs[ji].layer_numel[l]]

    def algorithmic_bytes(self) -> int:
        return sum((4 * s.W + 16) * s.n_params for s in self.specs)

    def n_params(self) -> int:
        return sum(s.n_params for s in self.specs)

    def close(self) -> None:
        torch.cuda.synchronize()
        self.svc.close()


class OracleService:
    """The same jobs replayed on the CPU oracle.  gen_device: where the seeded
    generator runs before values are brought to the host (the generator gives
    identical bits on every device; the GPU is only faster)."""

    def __init__(self, oracle_mod, specs: Sequence[wl.JobSpec], seed: int,
                 cap_elems: Optional[int] = None, gen_device="cpu"):
        self.orc, self.specs, self.seed, self.gen = oracle_mod, list(specs), seed, gen_device
        cap = cap_elems if cap_elems is not None else oracle_mod.BLOCK_CAP_ELEMS
        self.jobs = []
        for ji, s in enumerate(specs):
            j = oracle_mod.OracleJob(tuple(s.layer_numel), s.W, s.lr, s.momentum, s.wd, cap_elems=cap)
            for l, n in enumerate(s.layer_numel):
                j.p[l][:] = layer_values(seed, "param", (ji, l), n, s.param_std, self.gen).cpu().numpy()
            self.jobs.append(j)

    def block_grads(self, ji: int, b: int, rnd: int) -> List[np.ndarray]:
        layer, off, n = self.jobs[ji].blocks[b]
        s = self.specs[ji]
        return [layer_values(self.seed, "grad", (ji, w, rnd, layer), n, s.grad_std, self.gen,
                             start=off).cpu().numpy() for w in range(s.W)]

    def step(self, rnd: int, wave: Optional[Sequence[Tuple[int, int]]] = None) -> None:
        if wave is None:
            wave = self.orc.pack_wave(self.jobs)
        for ji, b in wave:
            self.jobs[ji].aggregate(b, self.block_grads(ji, b, rnd))
