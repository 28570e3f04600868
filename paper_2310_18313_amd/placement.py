"""Placement of the large flat buffers in HBM on MI355X.

Measured on MI355X (copy rates between 4 GiB pieces of the whole device memory): the 288 GiB of HBM3E behave
as three regions of 96 GiB.  Streams that a kernel walks at the same time run faster when they live
in different regions: a copy between regions reaches about 5 % more bandwidth than a copy inside one
region.  For the whole cast + Adam step at 13e9 parameters the gain is between 1 % and 5 %, and the slow
outliers of plain allocation (the first process on a freshly booted GPU) disappear.  What the kernels feel
is distance: with the buffers of a 1e9-parameter state carved out of one allocation, the update kernel runs
at 5.0 TB/s while they are within 8 GiB of each other, 5.8 TB/s at 16 GiB and 5.9-6.1 TB/s from 32 GiB on
(small offsets on top, from 4 KiB to hundreds of MiB, change nothing).  Buffers of 12 GiB and more are that
far apart by themselves; smaller ones, allocated one after the other, are not, and gain 10 % of the step
from this allocator.

`SpreadAllocator` therefore puts the buffers of an optimizer state into chosen regions without
assuming anything about the allocator: it takes all free device memory in slabs, finds out which
slabs share a region by timing copies between them, then frees exactly the slabs a buffer should
occupy and allocates the buffer into that hole.  The remaining slabs are released at the end.
For buffers smaller than a slab the memory that the slabs left over is taken as well, so that the
freed slab is the only place where such a buffer fits.  Where a buffer lands is still up to the
driver: in a process that has allocated and freed much before, small buffers have been seen to end
up next to each other all the same (then nothing is lost against plain allocation).

Nothing here computes anything of the method: it only decides where `torch.zeros` buffers land.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import torch

GiB = 1 << 30
_ROUND = 2 << 20          # torch hands large blocks to hipMalloc in multiples of 2 MiB


def _round_up(n: int, m: int = _ROUND) -> int:
    return (n + m - 1) // m * m


def copy_rate(ctx, src: torch.Tensor, dst: torch.Tensor, nbytes: int, reps: int = 3) -> float:
    """GB/s (read + write) of the library's 128-bit copy kernel between two device buffers."""
    ctx.copy_bytes(src, dst, nbytes)
    torch.cuda.synchronize()
    ctx.set_timing(True)
    ctx.get_timing()
    for _ in range(reps):
        ctx.copy_bytes(src, dst, nbytes)
    n, ms = ctx.get_timing()["copy"]
    ctx.set_timing(False)
    return 2 * nbytes / (ms / n * 1e-3) / 1e9


def verify_spread(ctx, a: torch.Tensor, b: torch.Tensor) -> dict:
    """Compares a copy inside buffer `a` with a copy from `a` to `b` (1 GiB each).  Buffers in different
    regions copy measurably faster than a buffer onto itself."""
    nb = min(GiB, a.numel() * a.element_size() // 2 // 16 * 16, b.numel() * b.element_size() // 16 * 16)
    half = nb // a.element_size()
    inside = copy_rate(ctx, a, a[half:], nb)
    across = copy_rate(ctx, a, b, nb)
    return {"inside_GBps": round(inside, 1), "across_GBps": round(across, 1), "distinct": across > 1.025 * inside}


class SpreadAllocator:
    """Allocates named buffers region by region (see the module docstring).

    `plan` lists, per region, the buffers to put there as (name, numel, dtype).  Works whatever the
    process allocated before, as long as most of the device memory is still free.  If the regions
    cannot be told apart, or the plan does not fit, everything is allocated plainly and `spread` is
    False.
    """

    def __init__(self, ctx, device: int = 0, slab_gib: int = 4, threshold: float = 1.025):
        self.ctx = ctx
        self.device = torch.device(f"cuda:{device}")
        self.slab_bytes = slab_gib * GiB
        self.threshold = threshold
        self.spread = False
        self.regions: List[List[int]] = []      # slab indices per discovered region
        self.where: Dict[str, int] = {}
        self.log: Dict[str, object] = {}

    # -- discovery ---------------------------------------------------------------------------------
    def _discover(self) -> List[torch.Tensor]:
        slabs: List[torch.Tensor] = []
        while torch.cuda.mem_get_info(self.device)[0] > self.slab_bytes + 3 * GiB:
            slabs.append(torch.empty(self.slab_bytes, dtype=torch.uint8, device=self.device))
        probe = min(2 * GiB, self.slab_bytes)
        unassigned = list(range(len(slabs)))
        regions: List[List[int]] = []
        scratch_ok = len(slabs) >= 6
        while scratch_ok and unassigned and len(regions) < 8:
            ref = unassigned[0]
            rest = unassigned[1:]
            if len(rest) < 2:
                regions.append([ref] + rest)
                break
            rates = sorted((copy_rate(self.ctx, slabs[ref], slabs[k], probe, reps=2), k) for k in rest)
            # Copies inside the reference's region are the slow ones.  Split the sorted rates in two
            # where the means of the two sides are furthest apart; accept the split only if the fast
            # side is clearly faster.
            vals = [r for r, _ in rates]
            best, cut = 1.0, None
            for i in range(1, len(vals)):
                lo, hi = sum(vals[:i]) / i, sum(vals[i:]) / (len(vals) - i)
                score = (hi - lo) * min(i, len(vals) - i) ** 0.25
                if cut is None or score > best:
                    best, cut = score, i
            lo, hi = sum(vals[:cut]) / cut, sum(vals[cut:]) / (len(vals) - cut)
            if hi >= self.threshold * lo:
                same = [ref] + [k for _, k in rates[:cut]]
            else:
                same = [ref] + rest              # no structure left: one region
            regions.append(sorted(same))
            unassigned = [k for k in unassigned if k not in same]
        self.regions = regions
        self.log["slabs"] = len(slabs)
        self.log["slab_GiB"] = self.slab_bytes // GiB
        self.log["region_slabs"] = [len(r) for r in regions]
        return slabs

    def _fill(self, keep_free: int) -> List[torch.Tensor]:
        """Takes what the slabs left over, in ever smaller blocks, until less than `keep_free` bytes are free.
        A buffer smaller than a slab would otherwise land in that remainder instead of in the slab freed
        for it."""
        fillers: List[torch.Tensor] = []
        try:
            for block in (GiB, 256 << 20, 64 << 20, 16 << 20):
                while torch.cuda.mem_get_info(self.device)[0] > keep_free + block and len(fillers) < 256:
                    fillers.append(torch.empty(block, dtype=torch.uint8, device=self.device))
        except RuntimeError:          # fragmented remainder: what has been taken is enough
            pass
        self.log["fillers"] = len(fillers)
        return fillers

    # -- allocation --------------------------------------------------------------------------------
    def allocate(self, plan: Sequence[Sequence[Tuple[str, int, torch.dtype]]]) -> Dict[str, torch.Tensor]:
        sizes = [[_round_up(n * torch.empty((), dtype=dt).element_size()) for _, n, dt in reg] for reg in plan]
        want = sum(sum(s) for s in sizes)
        smallest = min((b for s in sizes for b in s), default=0)
        free = torch.cuda.mem_get_info(self.device)[0]
        bufs: Dict[str, torch.Tensor] = {}
        slabs: List[torch.Tensor] = []
        fillers: List[torch.Tensor] = []
        ok = want >= 256 << 20 and smallest >= 32 << 20 and free > want + 16 * GiB and free > 64 * GiB
        if ok:
            slabs = self._discover()
            if smallest < self.slab_bytes:
                fillers = self._fill(max(16 << 20, smallest // 2))
            big = sorted((r for r in self.regions if len(r) >= 2), key=len, reverse=True)
            need = [-(-sum(s) // self.slab_bytes) for s in sizes]          # slabs per plan region
            ok = len(big) >= len(plan) and all(len(big[i]) >= need[i] for i in range(len(plan)))
        if not ok:
            del slabs, fillers
            torch.cuda.empty_cache()
            for reg in plan:
                for name, n, dt in reg:
                    bufs[name] = torch.zeros(n, dtype=dt, device=self.device)
                    self.where[name] = 0
            return bufs
        # heaviest plan region into the largest discovered region, and so on
        order = sorted(range(len(plan)), key=lambda i: -sum(sizes[i]))
        for rank, i in enumerate(order):
            take = big[rank][:need[i]]
            for k in take:
                slabs[k] = None                  # free exactly these slabs ...
            torch.cuda.empty_cache()
            for name, n, dt in plan[i]:          # ... and let the buffers fall into the hole
                bufs[name] = torch.zeros(n, dtype=dt, device=self.device)
                self.where[name] = rank
        del slabs, fillers
        torch.cuda.empty_cache()
        self.spread = True
        return bufs
