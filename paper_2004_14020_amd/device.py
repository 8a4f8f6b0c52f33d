"""Device memory plumbing (PyTorch): replica arenas, uploads, downloads.

No arithmetic of the method happens here; tensors are only containers whose
addresses are handed to the library.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from .binding import BF16, F32, Plan


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


class Replicas:
    """W replicas of a gradient set in device memory, one contiguous arena per replica.

    Tensor t of every replica starts at the same offset in its arena, like the flat gradient
    buffer of a training framework.  Tensors of at least `large_bytes` start on `large_align`
    boundaries (64 KiB: the reduce kernel's large tiles then coincide with aligned 64 KiB
    blocks of memory, which it streams measurably faster); the others on `slot_align`.
    Every arena starts at an address congruent to `arena_phase` (default 0, a multiple of 256
    below 64 KiB) modulo 2 MiB, so that tests can choose how runs sit relative to aligned blocks;
    `arena_phases`, one value per replica, places the replicas differently from one another."""

    def __init__(self, plan: Plan, elems: Sequence[int], device: str = "cuda:0", slot_align: int = 256,
                 large_align: int = 65536, large_bytes: int = 1 << 20,
                 with_workspace: bool = True, arena_phase: Optional[int] = None,
                 arena_phases: Optional[Sequence[int]] = None):
        self.plan = plan
        self.world = plan.cfg.world
        self.elems = [int(e) for e in elems]
        self.es = 4 if plan.cfg.dtype == F32 else 2
        self.np_dtype = np.float32 if plan.cfg.dtype == F32 else np.uint16
        self.torch_dtype = torch.float32 if plan.cfg.dtype == F32 else torch.int16
        self.device = torch.device(device)
        offs, at = [], 0
        for n in self.elems:
            at = _round_up(at, large_align if n * self.es >= large_bytes else slot_align)
            offs.append(at)
            at += n * self.es
        self.offsets = offs
        self.arena_bytes = max(at, slot_align)
        # Every arena starts at the same position inside an aligned 2 MiB block (position 0 unless
        # `arena_phase` says otherwise), as separately allocated flat buffers do; a caching
        # allocator that carves a new tensor out of a freed larger one does not promise that, so
        # the arenas are cut out of slightly larger tensors.
        phase = 0 if arena_phase is None else arena_phase
        if phase % 256 or not 0 <= phase < 65536:
            raise ValueError("arena_phase must be a multiple of 256 below 65536")
        block = 2 << 20
        self._backing = [torch.empty(self.arena_bytes + block, dtype=torch.uint8, device=self.device)
                         for _ in range(self.world)]
        self.arenas = []
        for w, b in enumerate(self._backing):
            ph = phase if arena_phases is None else int(arena_phases[w])
            if ph % 256 or not 0 <= ph < 65536:
                raise ValueError("arena phases must be multiples of 256 below 65536")
            skip = (ph - b.data_ptr()) % block
            self.arenas.append(b[skip:skip + self.arena_bytes])
        fe = plan.fused_elems
        self.fused: Optional[torch.Tensor] = None
        if with_workspace and fe > 0:
            self.fused = torch.empty(self.world * fe * self.es, dtype=torch.uint8, device=self.device)
        plan.bind(self.pointers(), self.fused.data_ptr() if self.fused is not None else None)

    def pointers(self) -> List[List[int]]:
        """Device address of every tensor of every replica, [worker][tensor]."""
        return [[a.data_ptr() + o for o in self.offsets] for a in self.arenas]

    def rebind(self) -> None:
        self.plan.bind(self.pointers(), self.fused.data_ptr() if self.fused is not None else None)

    def tensor(self, w: int, t: int) -> torch.Tensor:
        o, n = self.offsets[t], self.elems[t]
        return self.arenas[w][o:o + n * self.es].view(self.torch_dtype)

    def upload(self, grads: List[List[np.ndarray]]) -> None:
        for w in range(self.world):
            host = np.zeros(self.arena_bytes, dtype=np.uint8)
            for t, o in enumerate(self.offsets):
                src = np.ascontiguousarray(grads[w][t]).view(np.uint8)
                host[o:o + src.size] = src
            self.arenas[w].copy_(torch.from_numpy(host))
        torch.cuda.synchronize(self.device)

    def download(self) -> List[List[np.ndarray]]:
        torch.cuda.synchronize(self.device)
        out = []
        for w in range(self.world):
            host = self.arenas[w].cpu().numpy()
            out.append([host[o:o + n * self.es].view(self.np_dtype).copy()
                        for o, n in zip(self.offsets, self.elems)])
        return out

    def download_fused(self) -> Optional[np.ndarray]:
        if self.fused is None:
            return None
        torch.cuda.synchronize(self.device)
        return self.fused.cpu().numpy().view(self.np_dtype).reshape(self.world, -1).copy()

    def fill_fused(self, byte: int) -> None:
        if self.fused is not None:
            self.fused.fill_(byte)

    def fill_random(self, seed: int = 0) -> None:
        """Device-side fill for timing runs only (values do not affect speed)."""
        g = torch.Generator(device=self.device)
        g.manual_seed(seed)
        for w in range(self.world):
            n = self.arena_bytes // 4
            v = self.arenas[w][:n * 4].view(torch.float32)
            v.normal_(0.0, 1e-2, generator=g)
            if self.es == 2:
                # keep bf16 halves finite: clear the low exponent/mantissa mix of odd halves
                self.arenas[w][:n * 4].view(torch.int16).bitwise_and_(0x3FFF)
        torch.cuda.synchronize(self.device)
