"""Placement of the large flat buffers in HBM on MI355X.

Measured on MI355X (bench.py --region-map): the 288 GiB of HBM3E behave as three regions of 96 GiB of the physical
address space.  Streams that are only read do not care where they lie (6.7-7.0 TB/s anywhere).  Traffic that mixes
reads and writes -- the update pass reads and rewrites m, v and w in place -- reaches 5.2 TB/s while all of it falls
into one region and 6.3 TB/s once it is split over two or three of them, whatever the distance otherwise: the update
pass of a 13e9-parameter state takes 30 ms with its five streams in one region, 26.5 ms with all but the weight copy
in one region (what one plain allocation in the order v, gradient source, w, m, FP8 gradient, copy gives in a fresh
process, where device memory is handed out from the bottom of the address space upwards), and 24.5 ms when each
region carries about half of the bytes.

`RegionAllocator` therefore puts the buffers of an optimizer state into two groups that carry the same traffic in the
update pass -- (v, m, gradient source) and (w, FP8 gradient, weight copy) -- and makes sure the two groups lie in
different regions, by measurement and with bounded memory: it allocates the first group plainly, then steps through
device memory with 4 GiB spacers until a spacer lies in another region than the first group (told apart with the
library's update-shaped memory skeleton: 20 % faster across regions than inside one), allocates the second group
there, verifies head and tail of every buffer, and frees the spacers.  At most `max_spacer_gib` of spacers are held,
briefly; nothing else of the device is touched.  If the regions cannot be told apart, or the memory runs out, the
buffers stay where plain allocation put them and `spread` is False.

Nothing here computes anything of the method: it only decides where `torch.zeros` buffers land.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B

GiB = 1 << 30
REGION_GIB = 96           # what was measured; the allocator does not rely on it


def _bytes(t: torch.Tensor) -> torch.Tensor:
    return t.view(torch.uint8) if t.dtype != torch.uint8 else t


def probe_elems(a: torch.Tensor, b: torch.Tensor, cap: int = 1 << 29) -> int:
    """Largest element count (a multiple of a tile) the probe can run with its 16-bit streams in `a` and its 8-bit
    streams in `b`."""
    na, nb = a.numel() * a.element_size(), b.numel() * b.element_size()
    return min(cap, na // 4, nb // 3) // 4096 * 4096


def probe_ms(ctx, a: torch.Tensor, b: torch.Tensor, n: Optional[int] = None, reps: int = 3) -> float:
    """Time of the update-shaped memory skeleton (12 bytes per element, reads and writes mixed) with its two 16-bit
    streams in the first 4n bytes of `a` and its three 8-bit streams in the first 3n bytes of `b`.  Both buffers are
    overwritten with meaningless data.  The same `n` in different regions runs about 20 % faster than in one."""
    a, b = _bytes(a), _bytes(b)
    n = probe_elems(a, b) if n is None else n
    if n <= 0:
        raise ValueError("buffers too small for the probe")
    v, w = a[:2 * n].view(torch.int16), a[2 * n:4 * n].view(torch.int16)
    g, m, q = b[:n], b[n:2 * n], b[2 * n:3 * n]
    bufs = [g, m, v, w, q]
    ctx.memory_skeleton(B.SKEL_UPDATE, bufs, n)
    torch.cuda.synchronize()
    ctx.set_timing(True)
    ctx.get_timing()
    for _ in range(reps):
        ctx.memory_skeleton(B.SKEL_UPDATE, bufs, n)
    k, ms = ctx.get_timing()["skeleton"]
    ctx.set_timing(False)
    return ms / k


def verify_spread(ctx, a: torch.Tensor, b: torch.Tensor) -> dict:
    """Compares the probe inside buffer `a` with the probe across `a` and `b` (both are overwritten).  Buffers in
    different regions are clearly faster than a buffer against itself."""
    a, b = _bytes(a), _bytes(b)
    n = min(probe_elems(a[:a.numel() * 4 // 7], a[a.numel() * 4 // 7:]), probe_elems(a, b))
    inside = probe_ms(ctx, a[:4 * n], a[4 * n:7 * n], n)
    across = probe_ms(ctx, a[:4 * n], b, n)
    return {"elements": n, "inside_ms": round(inside, 4), "across_ms": round(across, 4), "distinct": across < 0.91 * inside}


class RegionAllocator:
    """Allocates two groups of named buffers into different HBM regions (see the module docstring).

    `plan` lists the two groups, each a list of (name, numel, dtype).  The first buffer of the first group is the
    anchor; every buffer of the second group is verified, head and tail, to lie in another region than the anchor;
    the remaining buffers of the first group are allocated last, plainly, into what the spacers leave behind.
    `where[name]`: 0 in the anchor's region, 1 in another one, 2 across a boundary, -1 not looked at.
    """

    def __init__(self, ctx, device: int = 0, spacer_gib: int = 4, max_spacer_gib: int = 200, ratio: float = 0.91):
        self.ctx = ctx
        self.device = torch.device(f"cuda:{device}")
        self.spacer_bytes = spacer_gib * GiB
        self.max_spacer_bytes = max_spacer_gib * GiB
        self.ratio = ratio
        self.spread = False
        self.where: Dict[str, int] = {}
        self.log: Dict[str, object] = {}

    def _zeros(self, n: int, dt: torch.dtype) -> torch.Tensor:
        return torch.zeros(n, dtype=dt, device=self.device)

    def allocate(self, plan: Sequence[Sequence[Tuple[str, int, torch.dtype]]]) -> Dict[str, torch.Tensor]:
        bufs: Dict[str, torch.Tensor] = {}
        first, second = list(plan[0]), list(plan[1])
        for name, _, _ in first + second:
            self.where[name] = -1
        spacers: List[torch.Tensor] = []
        torch.cuda.empty_cache()
        try:
            self.spread = self._place(bufs, first, second, spacers)
        except (RuntimeError, MemoryError) as e:          # out of memory on the way: what exists stays, the rest is plain
            self.log["gave_up"] = str(e).splitlines()[0][:120]
            self.spread = False
        self.log.setdefault("spacers_GiB", round(sum(t.numel() * t.element_size() for t in spacers) / GiB, 1))
        spacers.clear()
        torch.cuda.empty_cache()
        for name, _, _ in first:
            if name in bufs:
                bufs[name].zero_()                       # the probes wrote into them
        for name, n, dt in first + second:
            if name not in bufs:
                bufs[name] = self._zeros(n, dt)
        return bufs

    def _place(self, bufs, first, second, spacers) -> bool:
        size = lambda k, dt: k * torch.empty((), dtype=dt).element_size()
        a_name, a_k, a_dt = first[0]
        smallest = min(size(k, dt) for _, k, dt in [first[0]] + second)
        n = min(1 << 29, size(a_k, a_dt) // 7, smallest // 3) // 4096 * 4096   # the probe fits the anchor and every buffer
        if n < (1 << 27) or self.spacer_bytes < 3 * n:
            self.log["gave_up"] = "buffers too small for their place to matter"
            return False
        held = lambda: sum(t.numel() * t.element_size() for t in spacers)

        def room(nbytes: int) -> bool:
            return torch.cuda.mem_get_info(self.device)[0] > nbytes + 2 * GiB and held() <= self.max_spacer_bytes

        # 1. the anchor: a buffer whose head and tail lie in one region
        anchor = inside = None
        for _ in range(4):
            if not room(size(a_k, a_dt)):
                break
            t = _bytes(self._zeros(a_k, a_dt))
            t_in = probe_ms(self.ctx, t[:4 * n], t[4 * n:7 * n], n)
            t_tail = probe_ms(self.ctx, t[:4 * n], t[t.numel() - 3 * n:], n)
            if self.ratio * t_in <= t_tail <= t_in / self.ratio:
                anchor, inside = t, max(t_in, t_tail)
                break
            spacers.append(t)                            # head and tail in different regions: step over it
        if anchor is None:
            self.log["gave_up"] = "no anchor buffer inside one region"
            return False
        bufs[a_name] = anchor.view(a_dt)
        self.where[a_name] = 0
        head = anchor[:4 * n]
        self.log.update(probe_elements=n, inside_ms=round(inside, 4))

        def region_of(t: torch.Tensor) -> int:
            t = _bytes(t)
            h = probe_ms(self.ctx, head, t[:3 * n], n) < self.ratio * inside
            tl = probe_ms(self.ctx, head, t[t.numel() - 3 * n:], n) < self.ratio * inside
            return 1 if (h and tl) else 0 if not (h or tl) else 2

        # 2. step through memory until a spacer lies elsewhere, then allocate the second group and keep what verifies
        pending = list(second)
        across = []
        while pending:
            need = sum(size(k, dt) for _, k, dt in pending)
            if not room(need + self.spacer_bytes):
                self.log["gave_up"] = "another region not reached within the memory allowed"
                return False
            s = torch.empty(self.spacer_bytes, dtype=torch.uint8, device=self.device)
            spacers.append(s)
            t_ms = probe_ms(self.ctx, head, s, n)
            if t_ms >= self.ratio * inside:
                continue
            across.append(round(t_ms, 4))
            still = []
            for name, k, dt in pending:
                t = self._zeros(k, dt)
                r = region_of(t)
                if r == 1:
                    t.zero_()
                    bufs[name] = t
                    self.where[name] = 1
                else:
                    spacers.append(_bytes(t))            # a buffer in the wrong place is one more spacer
                    still.append((name, k, dt))
            pending = still
        self.log["across_ms"] = across[:4]
        # 3. the rest of the first group goes where the spacers were
        self.log["spacers_GiB"] = round(held() / GiB, 1)
        spacers.clear()
        torch.cuda.empty_cache()
        for name, k, dt in first[1:]:
            bufs[name] = self._zeros(k, dt)
            self.where[name] = region_of(bufs[name]) if size(k, dt) >= 3 * n else -1
        return True
