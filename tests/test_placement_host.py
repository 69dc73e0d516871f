"""Host logic of the region-aware placement (no GPU): region runs, carving through the library's
sgp_placer_* calls, fallbacks, roles."""
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
    for name, role in (("x", "x"), ("u", "u"), ("z", "z"), ("g0", "g"), ("g1", "g")):
        (off, nbytes), cls = p.floats(n, ld, role)
        got[name] = (off, nbytes, cls)
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
    offs0 = [p.floats(*one, "x")[0][0] // GIB for _ in range(8)]
    assert offs0[:4] == [1, 2, 3, 4]                           # interior of the 6-granule run
    assert sorted(offs0[4:6]) == [0, 5] and sorted(offs0[6:]) == [7, 8]   # its edges, then the short run
    offs1 = [p.floats(*one, "u")[0][0] // GIB for _ in range(6)]
    assert offs1[:3] == [10, 11, 12] and sorted(offs1[3:5]) == [9, 13] and offs1[5] == 6


def test_falls_back_to_another_region_when_one_is_full_and_raises_when_all_are():
    m = _map([0, 1], granule=1 * GIB)
    p = Placer(FakeArena(2 * GIB), m)
    big = (1, (GIB // 4) * 3 // 4)          # 0.75 GiB
    (_, _), c0 = p.floats(*big, "x")
    (_, _), c1 = p.floats(*big, "x")        # class 0 is full now
    assert {c0, c1} == {0, 1}
    with pytest.raises(MemoryError):
        p.floats(*big, "x")
    p.reset()                               # everything is free again
    (_, _), c2 = p.floats(*big, "x")
    assert c2 == c0


def test_single_class_map_still_carves_sequentially():
    m = _map([0, 0, 0], granule=1 * GIB)
    p = Placer(FakeArena(3 * GIB), m)
    offs = [p.floats(1, 1 << 20, role)[0][0] for role in ("x", "u", "z")]
    assert offs == [0, 4 << 20, 8 << 20]                       # a short run is used from its start


def test_smoothing_removes_isolated_outliers_and_renumbers():
    from paper_1811_10792_amd.binding import sgp_smooth_region_classes as smooth_classes
    raw = [0] * 12 + [1] * 4 + [2] + [1] * 7 + [3] * 11
    assert smooth_classes(raw) == [0] * 12 + [1] * 12 + [2] * 11
    assert smooth_classes([0, 0, 1, 1]) == [0, 0, 1, 1]          # a real boundary stays
    assert smooth_classes([2, 2, 0, 0]) == [0, 0, 1, 1]
    assert smooth_classes([0]) == [0] and smooth_classes([]) == []


def test_roles_share_and_separate_regions_as_documented():
    classes = [0] * 12 + [1] * 12 + [2] * 11
    p = Placer(FakeArena(len(classes) * 8 * GIB), _map(classes))
    arr = (16, 213_000_192)                                      # 13.6 GB each
    cls = {role: p.floats(*arr, role)[1] for role in ("x", "g", "u", "z", "msg0", "msg1", "v")}
    assert cls["g"] == cls["x"] == cls["v"] and cls["msg0"] == cls["msg1"] == cls["u"]
    assert len({cls["x"], cls["u"], cls["z"]}) == 3


def test_placer_argument_checks():
    import ctypes
    from paper_1811_10792_amd import binding
    lib = binding.load_library()
    out = ctypes.c_void_p()
    cls = (ctypes.c_int32 * 4)(0, 0, 1, 1)
    assert lib.sgp_placer_create(None, cls, 4, GIB) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_create(ctypes.byref(out), None, 4, GIB) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_create(ctypes.byref(out), cls, 0, GIB) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_create(ctypes.byref(out), cls, 4, GIB + 1) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_create(ctypes.byref(out), cls, 4, GIB) == binding.SGP_OK
    off, c = ctypes.c_int64(), ctypes.c_int32()
    assert lib.sgp_placer_take(out, 9, 4096, ctypes.byref(off), ctypes.byref(c)) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_take(out, 0, 0, ctypes.byref(off), ctypes.byref(c)) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_take(out, 0, 4096, None, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_placer_take(out, 0, 100, ctypes.byref(off), None) == binding.SGP_OK and off.value % 4096 == 0
    assert lib.sgp_placer_take(out, 0, 3 * GIB, ctypes.byref(off), ctypes.byref(c)) == binding.SGP_ERR_NOMEM
    assert lib.sgp_placer_destroy(out) == binding.SGP_OK and lib.sgp_placer_destroy(None) == binding.SGP_OK
