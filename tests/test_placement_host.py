"""Host logic of the region-aware placement (no GPU): region runs, carving, fallbacks."""
import pytest

from paper_1811_10792_amd.placement import GIB, Placer, RegionMap


class FakeArena:
    def __init__(self, nbytes):
        self.nbytes = nbytes

    def floats(self, offset_bytes, n, ld):
        assert offset_bytes % 4096 == 0 and offset_bytes + n * ld * 4 <= self.nbytes
        return (offset_bytes, n * ld * 4)


def _map(classes, granule=8 * GIB):
    return RegionMap(granule, list(classes), [], len(set(classes)) > 1)


def test_runs_and_capacity():
    m = _map([0, 0, 1, 1, 1, 0, 2, 2])
    assert m.runs(0) == [(0, 2), (5, 1)] and m.runs(1) == [(2, 3)] and m.runs(2) == [(6, 2)]
    assert m.capacity(1) == 3 * 8 * GIB and m.capacity(3) == 0


def test_written_streams_go_to_different_regions_and_never_overlap():
    classes = [0] * 12 + [1] * 12 + [2] * 11
    m = _map(classes)
    p = Placer(FakeArena(len(classes) * 8 * GIB), m)
    n, ld = 32, 25_557_248
    got = {}
    for role, want in (("x", 0), ("u", 1), ("z", 2), ("g0", 0), ("g1", 0)):
        (off, nbytes), cls = p.floats(n, ld, want)
        got[role] = (off, nbytes, cls)
    assert len({got[r][2] for r in ("x", "u", "z")}) == 3
    assert got["g0"][2] == got["x"][2] == got["g1"][2]
    spans = sorted((o, o + b) for o, b, _ in got.values())
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    for off, nbytes, cls in got.values():          # every array lies wholly inside its region,
        first, last = off // m.granule, (off + nbytes - 1) // m.granule
        assert all(m.classes[g] == cls for g in range(first, last + 1))
        assert all(m.classes[g - 1] == cls and m.classes[g + 1] == cls     # away from its edges
                   for g in range(first, last + 1))


def test_long_run_interiors_are_used_before_edges_and_short_runs():
    classes = [0] * 6 + [1] + [0] * 2 + [1] * 5
    m = _map(classes, granule=1 * GIB)
    p = Placer(FakeArena(len(classes) * GIB), m)
    one = (1, GIB // 4)                                        # exactly one granule
    offs0 = [p.floats(*one, 0)[0][0] // GIB for _ in range(8)]
    assert offs0[:4] == [1, 2, 3, 4]                           # interior of the 6-granule run
    assert sorted(offs0[4:6]) == [0, 5] and sorted(offs0[6:]) == [7, 8]   # its edges, then the short run
    offs1 = [p.floats(*one, 1)[0][0] // GIB for _ in range(6)]
    assert offs1[:3] == [10, 11, 12] and sorted(offs1[3:5]) == [9, 13] and offs1[5] == 6


def test_falls_back_to_another_region_when_one_is_full_and_raises_when_all_are():
    m = _map([0, 1], granule=1 * GIB)
    p = Placer(FakeArena(2 * GIB), m)
    big = (1, (GIB // 4) * 3 // 4)          # 0.75 GiB
    (_, _), c0 = p.floats(*big, 0)
    (_, _), c1 = p.floats(*big, 0)          # class 0 is full now
    assert {c0, c1} == {0, 1}
    with pytest.raises(MemoryError):
        p.floats(*big, 0)


def test_single_class_map_still_carves_sequentially():
    m = _map([0, 0, 0], granule=1 * GIB)
    p = Placer(FakeArena(3 * GIB), m)
    offs = [p.floats(1, 1 << 20, want)[0][0] for want in (0, 1, 2)]
    assert offs == [0, 4 << 20, 8 << 20]                       # a short run is used from its start


def test_smoothing_removes_isolated_outliers_and_renumbers():
    from paper_1811_10792_amd.binding import sgp_smooth_region_classes as smooth_classes
    raw = [0] * 12 + [1] * 4 + [2] + [1] * 7 + [3] * 11
    assert smooth_classes(raw) == [0] * 12 + [1] * 12 + [2] * 11
    assert smooth_classes([0, 0, 1, 1]) == [0, 0, 1, 1]          # a real boundary stays
    assert smooth_classes([2, 2, 0, 0]) == [0, 0, 1, 1]
    assert smooth_classes([0]) == [0] and smooth_classes([]) == []
