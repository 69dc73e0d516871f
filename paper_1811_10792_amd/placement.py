"""Placement of the state arrays inside HBM (host-side plumbing, no SGP arithmetic).

Measured on MI355X: the 288 GiB of HBM3E behave as three regions of 96 GiB (most likely the three
stack-ID ranks of the 12-high stacks), and concurrent streams that live in the SAME region slow
each other down (bank conflicts) while streams in different regions do not.  The fused step kernel
moves 3 read and 3 write streams for each of n nodes; with x, u and z in three different regions it
runs at 6.45 TB/s, with everything in one region at 5.2 TB/s.  A plain 1R+1W copy is hardly
affected (6.56 vs 6.68 TB/s).

User space cannot see physical addresses, so nothing is assumed about the map: one arena covering
most of the device memory is allocated, the regions are found by timing (`probe_regions`), and the
arrays are carved out of the arena so that the write streams land in different regions.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

GIB = 1 << 30


class Arena:
    """One large device allocation that arrays are carved out of (float32 views)."""

    def __init__(self, nbytes: int, device="cuda"):
        import torch
        self.nbytes = int(nbytes)
        self.buf = torch.empty(self.nbytes, dtype=torch.uint8, device=device)

    def floats(self, offset_bytes: int, n: int, ld: int):
        """float32 [n, ld] view starting `offset_bytes` into the arena (offset multiple of 4 KiB)."""
        import torch
        nbytes = n * ld * 4
        if offset_bytes % 4096 or offset_bytes < 0 or offset_bytes + nbytes > self.nbytes:
            raise ValueError("bad arena slice: offset %d, %d bytes" % (offset_bytes, nbytes))
        return self.buf[offset_bytes:offset_bytes + nbytes].view(torch.float32).view(n, ld)


@dataclass
class RegionMap:
    granule: int                 # bytes per probed granule
    classes: List[int]           # region class of every granule of the arena (-1 = not usable)
    times_ms: List[float]        # probe time of every granule in the first pass
    structured: bool             # False: no region structure was detected (single class)

    def runs(self, cls: int) -> List[Tuple[int, int]]:
        """Maximal runs (first granule, count) of granules of class `cls`."""
        out, start = [], None
        for i, c in enumerate(self.classes + [None]):
            if c == cls and start is None:
                start = i
            elif c != cls and start is not None:
                out.append((start, i - start))
                start = None
        return out

    def capacity(self, cls: int) -> int:
        return sum(1 for c in self.classes if c == cls) * self.granule


def smooth_classes(classes: List[int]) -> List[int]:
    """Regions are contiguous address ranges, so a single granule whose two neighbours agree with
    each other but not with it is a timing outlier: it takes its neighbours' class.  Classes are then
    renumbered in order of first appearance."""
    out = list(classes)
    for i in range(1, len(out) - 1):
        if out[i - 1] == out[i + 1] != out[i]:
            out[i] = out[i - 1]
    order: List[int] = []
    for c in out:
        if c not in order:
            order.append(c)
    return [order.index(c) for c in out]


def probe_regions(arena: Arena, granule: int = 8 * GIB, probe_d: int = 1 << 22, n: int = 32,
                  max_classes: int = 4) -> RegionMap:
    """Finds which granules of the arena interfere with each other.

    A small SGP problem (n nodes, probe_d coordinates) is stepped with x, u, g inside a reference
    granule and z inside the granule under test; a granule is in the reference's region when that
    step is slow.  Repeats with a new reference until every granule has a class.  Destroys the
    arena's contents.
    """
    from .binding import SGP
    count = arena.nbytes // granule
    arr = n * probe_d * 4
    if count < 2 or 4 * arr > granule:
        return RegionMap(granule, [0] * max(count, 1), [], False)
    eng = SGP(n, probe_d)
    eng.set_kernel_timing(True)
    import torch
    w = torch.ones(n, dtype=torch.float32, device=arena.buf.device)

    def time_with(ref: int, cand: int) -> float:
        base = ref * granule
        x, u, g = (arena.floats(base + j * arr, n, probe_d) for j in range(3))
        zoff = cand * granule + (3 * arr if cand == ref else 0)
        z = arena.floats(zoff, n, probe_d)
        for t in (x, u, g):
            t.zero_()
        w.fill_(1.0)
        for k in range(6):
            eng.step(x, w, u, g, z, 0.1, 0.9, k)
        ms = sorted(eng.step_kernel_times()[2:])
        return ms[len(ms) // 2]

    classes = [-1] * count
    first_times: List[float] = []
    structured = False
    for cls in range(max_classes):
        todo = [i for i in range(count) if classes[i] < 0]
        if not todo:
            break
        ref = todo[0]
        times = {i: time_with(ref, i) for i in todo}
        if cls == 0:
            first_times = [times[i] for i in range(count)]
        lo, hi = min(times.values()), max(times.values())
        if hi < 1.08 * lo:
            # no contrast: everything left behaves like the reference
            for i in todo:
                classes[i] = cls
            break
        structured = True
        mid = 0.5 * (lo + hi)
        for i in todo:
            if times[i] > mid:
                classes[i] = cls
        classes[ref] = cls
    for i in range(count):
        if classes[i] < 0:
            classes[i] = max_classes - 1
    eng.close()
    return RegionMap(granule, smooth_classes(classes), first_times, structured)


class Placer:
    """Hands out contiguous arena ranges inside a requested region class."""

    def __init__(self, arena: Arena, regions: RegionMap):
        self.arena, self.regions = arena, regions
        ncls = max(regions.classes) + 1
        # free ranges per class as [start_byte, end_byte), in the order they are tried: the interiors
        # of the long runs first, longest first (a granule at the edge of a run may straddle a region
        # boundary, and a short run may be a timing outlier), then what was trimmed off, then short runs
        g = regions.granule
        self.free: Dict[int, List[List[int]]] = {}
        for c in range(ncls):
            inner, edges, short = [], [], []
            for s0, k in sorted(regions.runs(c), key=lambda r: -r[1]):
                if k >= 4:
                    inner.append([(s0 + 1) * g, (s0 + k - 1) * g])
                    edges += [[s0 * g, (s0 + 1) * g], [(s0 + k - 1) * g, (s0 + k) * g]]
                else:
                    short.append([s0 * g, (s0 + k) * g])
            self.free[c] = inner + edges + short
        # classes ordered by capacity, largest first
        self.order = sorted(range(ncls), key=lambda c: -regions.capacity(c))

    def take(self, nbytes: int, cls: int) -> Optional[int]:
        """Byte offset of a fresh 4 KiB-aligned range of `nbytes` in class `cls`, or None."""
        need = (nbytes + 4095) // 4096 * 4096
        for run in self.free.get(cls, []):
            if run[1] - run[0] >= need:
                off = run[0]
                run[0] += need
                return off
        return None

    def floats(self, n: int, ld: int, want: int):
        """[n, ld] float32 tensor in the `want`-th largest region class (wrapping), falling back to
        any class with room."""
        tries = [self.order[(want + j) % len(self.order)] for j in range(len(self.order))]
        for cls in tries:
            off = self.take(n * ld * 4, cls)
            if off is not None:
                return self.arena.floats(off, n, ld), cls
        raise MemoryError("arena exhausted")


def make_placer(reserve_bytes: int = 6 * GIB, device="cuda", min_bytes: int = 0):
    """Allocates an arena over (almost) all free device memory and probes it.  Returns
    (placer, region_map), or (None, None) when the arena cannot be had (then allocate normally)."""
    import torch
    free, _total = torch.cuda.mem_get_info()
    granule = 8 * GIB
    nbytes = (free - reserve_bytes) // granule * granule
    if nbytes < max(min_bytes, 2 * granule):
        return None, None
    try:
        arena = Arena(nbytes, device)
    except RuntimeError:
        return None, None
    regions = probe_regions(arena, granule)
    return Placer(arena, regions), regions


class StateAllocator:
    """Allocates the [n, ld] float32 state arrays of one SGP problem, region-aware when an arena
    could be set up and plainly otherwise.  Roles: "x", "u", "z" are the three written streams and
    go to three different regions; "g" buffers are read-only and share the region of x; the
    message buffers of overlap mode go with u ("msg0") and with x ("msg1"): a message buffer written
    into the region of z measured 2.5 % slower (17.5 against 17.1 ms at n = 16, d = 213 M)."""

    ROLE_CLASS = {"x": 0, "g": 0, "u": 1, "msg0": 1, "z": 2, "msg1": 0, "v": 2}

    def __init__(self, mode: str = "regions", device="cuda"):
        self.device = device
        self.placer, self.regions = (make_placer(device=device) if mode == "regions" else (None, None))
        if self.placer is not None and not self.regions.structured:
            pass  # a single class: placement degenerates to sequential carving, still valid
        self.mode = "regions" if self.placer is not None else "default"
        self.placed: Dict[str, int] = {}

    def floats(self, role: str, n: int, ld: int, name: Optional[str] = None):
        import torch
        if self.placer is None:
            return torch.empty((n, ld), dtype=torch.float32, device=self.device)
        t, cls = self.placer.floats(n, ld, self.ROLE_CLASS[role])
        self.placed[name or role] = cls
        return t

    def reset(self) -> None:
        """Forgets every array handed out so far (their memory will be handed out again)."""
        if self.placer is not None:
            self.placer = Placer(self.placer.arena, self.regions)
        self.placed = {}

    def describe(self) -> dict:
        out = {"mode": self.mode}
        if self.regions is not None:
            out.update({"granule_gib": self.regions.granule // GIB,
                        "region_of_granule": "".join(str(c) for c in self.regions.classes),
                        "structured": self.regions.structured, "arrays": dict(self.placed)})
        return out
