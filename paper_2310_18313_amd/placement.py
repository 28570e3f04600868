"""Placement of the large flat buffers in HBM on MI355X.

Measured on MI355X (bench.py --region-map): the 288 GiB of HBM3E behave as three regions of 96 GiB of the physical
address space.  Streams that are only read do not care where they lie (6.7-7.1 TB/s anywhere).  Traffic that mixes
reads and writes -- the update pass reads and rewrites m, v and w in place -- reaches 5.2 TB/s while all of it falls
into one region and 6.2-6.3 TB/s once it is split over two or three of them, whatever the distance otherwise: the
update pass of a 13e9-parameter state takes 30 ms with its five streams in one region, 27 ms with all but an 8-bit
stream in one region and 24.5 ms when no region carries more than about four fifths of the bytes.  Where an allocation
lands is up to the driver: a large one is built from big physical blocks that need not be neighbours (a 120 GiB
allocation was seen as 64 GiB in one region, 32 GiB in another and 24 GiB in the first again), and what earlier
processes left behind changes the picture from one process to the next.  Only measurement tells.

`RegionAllocator` therefore keeps a tally of the update pass's traffic per region while it allocates, by measurement
and with bounded memory.  All kernels walk their buffers in step, so the tally is kept per place: seven places spread
evenly from head to tail of every buffer.  The anchor (v) is allocated first (again, up to three times, if it does not
lie in one region as a whole) and a window of it that lies inside one region becomes the reference.  Every further
buffer that the update pass touches is allocated plainly and looked up at its seven places against the reference
with the library's update-shaped memory skeleton (16 % faster across regions than inside one); at each place the
bytes per element that the update pass moves through the buffer are added to the reference's region or to the rest.
A buffer that would push the reference's region above two thirds of the traffic at any place (four fifths once
110 GiB of spacers are held) is kept aside as a spacer and allocated again, further on; one that only pushes the rest
above four fifths is kept, because stepping on rarely leads back into the region.  The spacers are freed at the end.  At most
`max_spacer_gib` of them are held, briefly; nothing else of the device is touched.  If no reference can be found or
memory runs short the buffers stay where plain allocation put them and `spread` is False.

A kernel that writes a single buffer (the cast writes the FP8 gradient) is limited by the region that buffer lies in,
whatever its reads do: 5.4 TB/s for the cast's two-to-one mix, against 6.0 TB/s when the written buffer itself alternates
between regions.  `StripedArena` builds such a buffer from 1 GiB pieces of device memory (HIP virtual memory
management through the library's fp8lm_vmm_* calls): pieces are created one by one and timed against the first, and
those kept are mapped into one address range in alternating order.

Nothing here computes anything of the method: it only decides where buffers land.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B

GiB = 1 << 30
REGION_GIB = 96           # what was measured; the allocator does not rely on it
# The probe moves 12 bytes per element: 5.2e12 B/s inside one region, 6.2e12 B/s across two.  A buffer whose own first
# bytes already run faster than this is made of pieces from several regions (small allocations in a process that has
# allocated and freed much) and cannot serve as the anchor.
MIXED_ABOVE_BPS = 5.5e12


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


def fits(here: Sequence[float], away: Sequence[float], weight: float, outside: Sequence[bool], lim_here: float,
         lim_away: float) -> bool:
    """The acceptance rule: `here[i]` / `away[i]` is the traffic already placed in / outside the reference's region at
    place i; a buffer of `weight` bytes per element that lies outside the region where `outside[i]` is accepted if
    no place ends up above its limit on either side."""
    return all((here[i] + weight <= lim_here) if not outside[i] else (away[i] + weight <= lim_away)
               for i in range(len(outside)))


class RegionAllocator:
    """Allocates named buffers so that neither the reference's region nor the rest of the device carries more than
    `limit` of a kernel's mixed traffic (`soft_limit` once `patience_gib` of spacers are held; beyond four fifths a
    region becomes the bottleneck).  See the module docstring.

    `plan`: (name, numel, dtype, weight) per buffer in the order of allocation, weight = bytes per element that the
    update pass moves through it (0: the buffer lies where it falls).  The first entry is the anchor.
    `where[name]`: per place looked at, from head to tail, 0 in the reference's region, 1 outside (None: not looked at).
    """

    def __init__(self, ctx, device: int = 0, max_spacer_gib: int = 200, limit: float = 0.67, soft_limit: float = 0.8,
                 patience_gib: int = 110, ratio: float = 0.91):
        self.ctx = ctx
        self.device = torch.device(f"cuda:{device}")
        self.max_spacer_bytes = max_spacer_gib * GiB
        self.limit = limit                  # share of the traffic one side may carry ...
        self.soft_limit = soft_limit        # ... and once more than patience_gib of spacers are held
        self.patience_bytes = patience_gib * GiB
        self.positions = 7                  # places per buffer at which its region is looked up
        self.ratio = ratio
        self.spread = False
        self.where: Dict[str, Optional[str]] = {}
        self.log: Dict[str, object] = {}

    def _zeros(self, n: int, dt: torch.dtype) -> torch.Tensor:
        return torch.zeros(n, dtype=dt, device=self.device)

    def allocate(self, plan: Sequence[Tuple[str, int, torch.dtype, float]], even_weight: float = 0.0) -> Dict[str, torch.Tensor]:
        """`even_weight`: bytes per element the update pass moves through buffers that are not in the plan because
        they lie evenly over the regions anyway (a StripedArena); counted half and half."""
        self.even_weight = float(even_weight)
        bufs: Dict[str, torch.Tensor] = {}
        for name, _, _, _ in plan:
            self.where[name] = None
        spacers: List[torch.Tensor] = []
        torch.cuda.empty_cache()
        try:
            self.spread = self._place(bufs, list(plan), spacers)
        except (RuntimeError, MemoryError) as e:          # out of memory on the way: what exists stays, the rest is plain
            self.log["gave_up"] = str(e).splitlines()[0][:120]
            self.spread = False
        self.log["spacers_GiB"] = round(sum(t.numel() * t.element_size() for t in spacers) / GiB, 1)
        spacers.clear()
        torch.cuda.empty_cache()
        for t in bufs.values():
            t.zero_()                                    # the probes wrote into them
        for name, n, dt, _ in plan:
            if name not in bufs:
                bufs[name] = self._zeros(n, dt)
        return bufs

    def _place(self, bufs, plan, spacers) -> bool:
        size = lambda k, dt: k * torch.empty((), dtype=dt).element_size()
        a_name, a_k, a_dt, a_w = plan[0]
        n = min(1 << 29, size(a_k, a_dt) // 7, min(size(k, dt) for _, k, dt, w in plan if w > 0) // 3) // 4096 * 4096
        if n < (1 << 27):
            self.log["gave_up"] = "buffers too small for their place to matter"
            return False
        total_w = float(sum(w for _, _, _, w in plan)) + self.even_weight
        K = self.positions
        held = lambda: sum(t.numel() * t.element_size() for t in spacers)

        def room(nbytes: int) -> bool:
            return torch.cuda.mem_get_info(self.device)[0] > nbytes + 2 * GiB and held() <= self.max_spacer_bytes

        def reference_in(anchor: torch.Tensor):
            """A window of the anchor that lies in one region (the probe inside it runs slowly): (window, ms, offset)."""
            for o in range(0, anchor.numel() - 7 * n + 1, 7 * n)[:8]:
                t_in = probe_ms(self.ctx, anchor[o:o + 4 * n], anchor[o + 4 * n:o + 7 * n], n)
                if 12 * n / (t_in * 1e-3) < MIXED_ABOVE_BPS:
                    return anchor[o:o + 4 * n], t_in, o
            return None, None, None

        def profile(t: torch.Tensor, ref, inside, skip=None) -> List[bool]:
            """At K places spread evenly over the buffer, head and tail included: does it lie outside the
            reference's region?  All kernels walk their buffers in step, so what has to be balanced is the traffic
            at each place, not its sum over the buffer."""
            t = _bytes(t)
            last = t.numel() - 3 * n
            out = []
            for i in range(K):
                o = (last * i // (K - 1)) // 4096 * 4096
                if skip is not None and o < skip + 7 * n and o + 3 * n > skip:
                    out.append(False)                    # overlaps the reference: its region by construction
                else:
                    out.append(probe_ms(self.ctx, ref, t[o:o + 3 * n], n, reps=2) < self.ratio * inside)
            return out

        # 1. the anchor, preferably a buffer that lies in one region as a whole
        anchor = ref = inside = prof = None
        for attempt in range(3):
            if not room(size(a_k, a_dt)):
                break
            t = _bytes(self._zeros(a_k, a_dt))
            r, t_in, at = reference_in(t)
            p = profile(t, r, t_in, skip=at) if r is not None else None
            if anchor is None or (p is not None and (prof is None or sum(p) < sum(prof))):
                if anchor is not None:
                    spacers.append(anchor)
                anchor, ref, inside, prof = t, r, t_in, p
            else:
                spacers.append(t)
            if prof is not None and not any(prof):
                break
        if anchor is None or ref is None:
            if anchor is not None:
                bufs[a_name] = anchor.view(a_dt)
            self.log["gave_up"] = "no window of the anchor lies inside one region (allocations come in small pieces from several)"
            return False
        bufs[a_name] = anchor.view(a_dt)
        self.where[a_name] = "".join("01"[x] for x in prof)
        self.log.update(probe_elements=n, inside_ms=round(inside, 4))
        here = [a_w * (not x) + self.even_weight / 2 for x in prof]      # traffic in the reference's region, at each place
        away = [a_w * x + self.even_weight / 2 for x in prof]
        # 2. every other buffer: keep it if neither side exceeds its limit at any place.  Too much in the reference's
        # region: step over the buffer, which leads out of the region sooner or later.  Too much outside it only:
        # stepping on rarely leads back, so the buffer is kept as it is.
        over = []
        for name, k, dt, w in plan[1:]:
            while True:
                if torch.cuda.mem_get_info(self.device)[0] < size(k, dt) + 2 * GiB:
                    raise MemoryError(f"no memory left for {name}")      # the caller frees the spacers and goes on plainly
                t = self._zeros(k, dt)
                if w <= 0:                               # not touched by the update pass: it lies where it falls
                    p = profile(t, ref, inside) if size(k, dt) >= 3 * n else []
                    break
                p = profile(t, ref, inside)
                lim_here = (self.limit if held() < self.patience_bytes else self.soft_limit) * total_w + 1e-9
                lim_away = self.soft_limit * total_w + 1e-9
                if fits(here, away, w, p, lim_here, lim_away):
                    break
                if fits(here, away, w, p, lim_here, float("inf")) or not room(size(k, dt)):
                    over.append(name)                    # nothing to gain, or nothing left to try with
                    break
                spacers.append(_bytes(t))                # in the wrong place: one more spacer
            bufs[name] = t
            self.where[name] = "".join("01"[x] for x in p) if p else None
            if w > 0:
                here = [here[i] + w * (not p[i]) for i in range(K)]
                away = [away[i] + w * p[i] for i in range(K)]
        if over:
            self.log["kept_over_the_limit"] = over
        # what counts in the end: the busiest side at the worst place, and on average over the places
        self.log["traffic_share_busiest"] = round(max(here + away) / total_w, 3)
        self.log["traffic_share_busiest_mean"] = round(sum(max(h, a) for h, a in zip(here, away)) / (K * total_w), 3)
        return self.log["traffic_share_busiest_mean"] <= self.soft_limit


class _Mappings:
    """Owns pieces of device memory mapped one after the other into a reserved address range; gives everything back
    when the last reference goes (after waiting for the device)."""

    def __init__(self, device: int, piece: int, nbytes: int):
        self.device, self.piece, self.nbytes = device, piece, nbytes
        self.va = B.vmm_reserve(nbytes)
        self.pieces: List[int] = []

    def append(self, handle: int) -> int:
        """Maps one more piece behind the pieces already there; returns its index."""
        k = len(self.pieces)
        B.vmm_map(self.va + k * self.piece, self.piece, handle, self.device)
        self.pieces.append(handle)
        return k

    def release(self, keep=()) -> None:
        """Unmaps everything; destroys the pieces not listed in `keep`; gives the range back."""
        if self.pieces:
            B.vmm_unmap(self.va, len(self.pieces) * self.piece)
        for h in self.pieces:
            if h not in keep:
                B.vmm_destroy(h)
        self.pieces = []
        if self.va:
            B.vmm_free(self.va, self.nbytes)
            self.va = 0

    def __del__(self):
        try:
            self.release()
        except Exception:           # interpreter shutdown, or the runtime is already gone
            pass


class _DeviceRange:
    """A range of device addresses as something torch can wrap without copying (and keep alive)."""

    def __init__(self, owner: _Mappings):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": (owner.nbytes,), "typestr": "|u1", "data": (owner.va, False),
                                         "version": 2, "strides": None}


class StripedArena:
    """One range of device addresses whose pieces alternate between two HBM regions (see the module docstring).

    Pieces of `piece_gib` are created one after the other, each mapped into a staging range and timed against the
    first piece with the update-shaped probe, until half of the bytes asked for can come from the first piece's
    region and half from elsewhere (in a fresh process that means creating pieces up to the next region; the ones
    not needed are destroyed at once).  The pieces kept are then mapped into one range in alternating order;
    `bytes` is that range as a tensor (zeroed) and `tensor(offset, nbytes, dtype)` hands out views of it, which keep
    the memory alive.  Raises RuntimeError (Fp8lmError is one) if the device has no virtual memory management, memory
    runs short, or fewer than `min_share` of the bytes can come from a second region.  `alternate=False` maps the first
    region's pieces first and the others after them (for measurements: same pieces, no alternation).
    """

    def __init__(self, ctx, nbytes: int, device: int = 0, piece_gib: float = 1.0, min_share: float = 0.25,
                 max_extra_gib: int = 160, alternate: bool = True):
        gran = B.vmm_granularity(device)
        piece = max(gran, int(piece_gib * GiB) // gran * gran)
        n = (nbytes + piece - 1) // piece
        n_probe = min(1 << 28, piece // 4) // 4096 * 4096
        if n < 4 or n_probe < (1 << 26):
            raise RuntimeError("too small for its place to matter")
        self.log: Dict[str, object] = {}
        want_away = n // 2
        limit = n + int(max_extra_gib * GiB) // piece
        staging = _Mappings(device, piece, limit * piece)
        is_away: List[bool] = []
        try:
            view = torch.as_tensor(_DeviceRange(staging), device=f"cuda:{device}")
            inside = None
            while (is_away.count(False) < n - want_away or is_away.count(True) < want_away) and len(is_away) < limit:
                if torch.cuda.mem_get_info(device)[0] < piece + 2 * GiB:
                    break
                k = staging.append(B.vmm_create(piece, device))
                if k == 0:
                    is_away.append(False)
                    continue
                t = probe_ms(ctx, view[:piece], view[k * piece:(k + 1) * piece], n_probe, reps=2)
                if inside is None and 12 * n_probe / (t * 1e-3) < MIXED_ABOVE_BPS:
                    inside = t                       # the first piece against a neighbour in its own region: slow
                is_away.append(inside is None or t < 0.91 * inside)
            del view
            handles = list(staging.pieces)
            away = [h for h, a in zip(handles, is_away) if a][:want_away]
            here = [h for h, a in zip(handles, is_away) if not a][:n - len(away)]
            self.log.update(piece_MiB=piece >> 20, pieces_created=len(handles), pieces_used=n,
                            created_outside_first_region=sum(is_away),
                            inside_ms=None if inside is None else round(inside, 4))
            if len(here) + len(away) < n or len(away) < min_share * n:
                raise RuntimeError(f"{len(away)} of the {n} pieces needed lie outside the first piece's region")
            staging.release(keep=here + away)
        except BaseException:
            staging.release()
            raise
        # the smaller group spread evenly through the larger one
        final = _Mappings(device, piece, n * piece)
        try:
            a = b = 0
            for _ in range(n):
                if b < len(away) and (a >= len(here) or (alternate and b * len(here) <= a * len(away))):
                    final.append(away[b])
                    b += 1
                else:
                    final.append(here[a])
                    a += 1
        except BaseException:
            mapped = set(final.pieces)
            final.release()
            for h in here + away:
                if h not in mapped:
                    B.vmm_destroy(h)
            raise
        self.log["share_outside_first_region"] = round(len(away) / n, 3)
        self.nbytes = n * piece
        self.bytes = torch.as_tensor(_DeviceRange(final), device=f"cuda:{device}")
        self.bytes.zero_()

    def tensor(self, offset: int, nbytes: int, dtype: torch.dtype = torch.uint8) -> torch.Tensor:
        return self.bytes[offset:offset + nbytes].view(dtype)
