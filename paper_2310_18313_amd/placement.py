"""Placement of the large flat buffers in HBM on MI355X.

Measured on MI355X (see `python -m paper_2310_18313_amd.placement --probe`): the 288 GiB of HBM3E behave
as three regions of 96 GiB each.  Streams that a kernel walks at the same time run faster when they
live in different regions (a copy between regions reaches about 5 % more bandwidth than a copy inside
one region; the eight-stream Adam update kernel about 18 % more).  A fresh process receives physical
memory in allocation order, so the regions can be targeted by allocating the buffers in a chosen
order with temporary ballast in between; the ballast is freed again once everything is placed.

Nothing here computes anything of the method: it only decides where `torch.zeros` buffers land.
"""
from __future__ import annotations

import sys
from typing import Dict, List, Sequence, Tuple

import torch

GiB = 1 << 30
N_REGIONS = 3
_ROUND = 2 << 20          # torch hands large blocks to hipMalloc in multiples of 2 MiB


def _round_up(n: int, m: int = _ROUND) -> int:
    return (n + m - 1) // m * m


class SpreadAllocator:
    """Allocates named buffers region by region.

    `plan` lists, per region, the buffers to put there as (name, numel, dtype).  Must be used before the
    process has made other large device allocations (the physical position is inferred from the amount
    of memory in use).  If the plan does not fit, or the device does not look like a 3 x 96 GiB
    MI355X, everything is allocated plainly and `spread` is False.
    """

    def __init__(self, device: int = 0):
        self.device = torch.device(f"cuda:{device}")
        free, total = torch.cuda.mem_get_info(self.device)
        self.total = total
        self.used0 = total - free
        self.region = total // N_REGIONS
        self.spread = False
        self.where: Dict[str, int] = {}

    def allocate(self, plan: Sequence[Sequence[Tuple[str, int, torch.dtype]]]) -> Dict[str, torch.Tensor]:
        sizes = [[_round_up(n * torch.empty((), dtype=dt).element_size()) for _, n, dt in reg] for reg in plan]
        want = sum(sum(s) for s in sizes)
        fits = (len(plan) <= N_REGIONS and abs(self.total - 288 * GiB) < 8 * GiB and want >= 2 * GiB and
                all(sum(s) <= self.region - (self.used0 if r == 0 else 0) - 64 * (1 << 20) for r, s in enumerate(sizes)))
        bufs: Dict[str, torch.Tensor] = {}
        ballast: List[torch.Tensor] = []
        pos = self.used0
        for r, reg in enumerate(plan):
            for (name, n, dt), nbytes in zip(reg, sizes[r]):
                bufs[name] = torch.zeros(n, dtype=dt, device=self.device)
                self.where[name] = r if fits else 0
                pos += nbytes
            end = (r + 1) * self.region
            if fits and r + 1 < len(plan) and pos < end:
                ballast.append(torch.empty(end - pos, dtype=torch.uint8, device=self.device))
                pos = end
        del ballast
        if fits:
            torch.cuda.empty_cache()
        self.spread = fits
        return bufs


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


def probe(piece_gib: int = 4) -> None:
    """Prints the copy rate from the first piece of device memory to every other piece."""
    from . import binding as B
    ctx = B.Context([(0, 16)])
    pieces = []
    free, total = torch.cuda.mem_get_info()
    print(f"total {total / GiB:.2f} GiB, free {free / GiB:.2f} GiB, piece {piece_gib} GiB", flush=True)
    while torch.cuda.mem_get_info()[0] > (piece_gib + 2) * GiB:
        pieces.append(torch.zeros(piece_gib * GiB, dtype=torch.uint8, device="cuda:0"))
    nb = min(piece_gib, 1) * GiB
    for ref in (0, len(pieces) // 2, len(pieces) - 1):
        print(f"copy of 1 GiB from piece {ref} (starts at about {ref * piece_gib} GiB) to piece k, GB/s:")
        row = []
        for k, p in enumerate(pieces):
            row.append("  ref" if k == ref else f"{copy_rate(ctx, pieces[ref], p, nb):5.0f}")
            if len(row) == 12 or k == len(pieces) - 1:
                print(" ".join(row) + f"   | up to {(k + 1) * piece_gib} GiB", flush=True)
                row = []


if __name__ == "__main__":
    if "--probe" in sys.argv:
        probe()
