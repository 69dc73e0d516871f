"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments, and its integer peer scheduler agrees bit for bit with the
positions of the non-zeros of the oracle's dense mixing matrix."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import sgp_oracle as O
import paper_1811_10792_amd as sgp
from paper_1811_10792_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1811_10792_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "sgp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sgp_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert binding.status_string(0) == "SGP_OK"
    names = {binding.status_string(c) for c in range(-6, 1)}
    assert len(names) == 7 and all(s.startswith("SGP_") for s in names)
    assert binding.status_string(-99) == "SGP_ERR_UNKNOWN"


def test_create_validates_arguments(lib):
    h = ctypes.c_void_p()
    ok = lambda *a: lib.sgp_create(ctypes.byref(h), *a)
    assert ok(4, 16, 16, 0, 1, 0) == 0 and h.value
    assert lib.sgp_destroy(h) == 0
    for bad in ((0, 16, 16, 0, 1, 0), (4, 0, 16, 0, 1, 0), (4, 16, 8, 0, 1, 0), (4, 16, 16, 0, 0, 0),
                (4, 16, 16, 0, 17, 0), (4, 16, 16, 0, 1, 65), (4, 16, 16, 0, 1, -1), (1025, 16, 16, 0, 1, 0)):
        assert ok(*bad) == binding.SGP_ERR_INVALID_ARG and not h.value
    assert ok(4, 16, 16, 7, 1, 0) == binding.SGP_ERR_UNSUPPORTED
    assert ok(4, 16, 16, 0, 1, 64) == 0 and lib.sgp_destroy(h) == 0
    assert lib.sgp_create(None, 4, 16, 16, 0, 1, 0) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_destroy(None) == 0


def test_null_pointers_are_rejected_before_any_launch(lib):
    h = ctypes.c_void_p()
    assert lib.sgp_create(ctypes.byref(h), 4, 16, 16, 0, 1, 0) == 0
    assert lib.sgp_step(h, None, None, None, None, None, 0.1, 0.9, 0, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_step(None, 16, 16, 16, 16, None, 0.1, 0.9, 0, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_step(h, 16, 16, None, 16, None, 0.1, 0.9, 0, None) == binding.SGP_ERR_INVALID_ARG  # momentum without m
    assert lib.sgp_step(h, 16, 16, 16, 16, None, 0.1, 0.9, -1, None) == binding.SGP_ERR_INVALID_ARG  # k < 0
    assert lib.sgp_step(h, 18, 16, 16, 16, None, 0.1, 0.9, 0, None) == binding.SGP_ERR_ALIGNMENT
    assert lib.sgp_debias(h, None, None, None, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_consensus_stats(h, None, None, None, None, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_copy(None, None, 16, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_copy(16, 32, 8, None) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_destroy(h) == 0


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built HIP library nothing runs: no CPU path stands in for it."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libsgp_hip.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        sgp.SGP(4, 16)


def test_every_translation_unit_is_built_and_every_declared_walk_variant_has_an_object():
    """build.py compiles each .hip file of csrc/, and the walk with fused statistics once for every
    variant whose launcher csrc/internal.h declares (a missing object would only show up as an
    undefined symbol when the library is loaded)."""
    import glob
    from paper_1811_10792_amd import build
    csrc = os.path.join(os.path.dirname(build.__file__), "csrc")
    sources = {os.path.basename(f) for f in glob.glob(os.path.join(csrc, "*.hip"))}
    assert {src for src, _, _ in build.UNITS} == sources
    assert len({name for _, name, _ in build.UNITS}) == len(build.UNITS)          # distinct objects
    declared = set()
    for m in re.finditer(r"^SGP_DECLARE_WALK_STATS\((\w+), (\w+), (\w+)\)", open(os.path.join(csrc, "internal.h")).read(),
                         re.M):
        nest, cached, msg = m.groups()
        declared.add((int(nest == "true"), int(cached == "true"), int(msg)))
    built = set()
    for src, _, defs in build.UNITS:
        if src == "sgp_walk_stats.hip":
            d = dict(x[2:].split("=") for x in defs)
            built.add((int(d["SGP_WALK_NEST"]), int(d["SGP_WALK_CACHED"]), int(d["SGP_WALK_MSG"])))
    assert built == declared and len(built) == 8


def test_stream_pattern_argument_checks(lib):
    """All of these are refused before anything is launched (the addresses are never touched)."""
    vp = ctypes.c_void_p

    def call(reads, writes, nbytes):
        r = (vp * max(1, len(reads)))(*reads)
        w = (vp * max(1, len(writes)))(*writes)
        return lib.sgp_stream_pattern(r, len(reads), w, len(writes), nbytes, None)
    bad = binding.SGP_ERR_INVALID_ARG
    assert call([], [], 1024) == bad                                   # nothing to do
    assert call([4096] * 5, [], 1024) == bad                           # more than four of a kind
    assert call([4096], [8192], 1000) == bad                           # not a multiple of 16
    assert call([4096], [8200], 1024) == bad                           # misaligned
    assert call([4096], [None], 1024) == bad
    assert call([4096], [4096 + 512], 1024) == bad                     # partial overlap of a read and a write
    assert call([4096], [16384, 16384], 1024) == bad                   # the same array written twice
    assert call([4096], [16384, 16384 + 512], 1024) == bad             # overlapping writes
    assert call([4096], [4096], 0) == 0                                # in place is fine; empty: nothing launched
    assert lib.sgp_stream_pattern(None, 1, None, 0, 1024, None) == bad


@pytest.mark.parametrize("peers", [1, 2, 3])
def test_schedule_matches_oracle_nonzeros_exactly(lib, peers):
    for n in list(range(1, 18)) + [31, 32, 33, 64, 100]:
        L = (n - 1).bit_length()
        for k in list(range(0, 2 * L + 2)) + [10 ** 6 + 3, 2 ** 40 + 5]:
            outp, inp, wt = sgp.sgp_schedule(n, peers, k)
            P32 = O.mixing_matrix(n, peers, k, np.float32)
            for i in range(n):
                senders_to = {j for j in outp[i] if j >= 0} | {i}
                hears_from = {j for j in inp[i] if j >= 0} | {i}
                assert senders_to == set(np.nonzero(P32[:, i])[0].tolist())   # column i: receivers
                assert hears_from == set(np.nonzero(P32[i, :])[0].tolist())   # row i: senders
            assert np.float32(wt) == P32[0, 0]                               # same float32 bits
            assert set(np.unique(P32[P32 != 0]).tolist()) == {float(np.float32(wt))}


def test_schedule_slots_and_duplicates(lib):
    outp, inp, wt = sgp.sgp_schedule(8, 2, 1)            # hops 2 and 4
    assert outp[0] == [2, 4] and inp[0] == [6, 4] and wt == np.float32(1.0) / np.float32(3.0)
    outp, inp, wt = sgp.sgp_schedule(2, 2, 0)            # the only peer, reached twice
    assert outp == [[1, -1], [0, -1]] and wt == 0.5
    outp, inp, wt = sgp.sgp_schedule(1, 1, 4)
    assert outp == [[-1]] and inp == [[-1]] and wt == 1.0
    # printed example: 8 nodes, node 0 sends to 1, 2, 4 over iterations 0, 1, 2, then wraps
    assert [sgp.sgp_schedule(8, 1, k)[0][0][0] for k in range(4)] == [1, 2, 4, 1]


def test_handle_schedule_equals_handle_free(lib):
    s = sgp.SGP(12, 40, peers=2)
    for k in range(9):
        assert s.peer_schedule(k) == sgp.sgp_schedule(12, 2, k)
    s.close()


def test_schedule_of_tau_overlap_advances_once_per_round(lib):
    """delay >= 2: peers only at k % delay == 0, and round c = k / delay uses schedule entry c."""
    n, peers, tau = 8, 2, 3
    h = ctypes.c_void_p()
    assert lib.sgp_create(ctypes.byref(h), n, 16, 16, 0, peers, tau) == 0
    out = (ctypes.c_int32 * (n * peers))()
    inp = (ctypes.c_int32 * (n * peers))()
    wt = ctypes.c_float()
    for k in range(4 * tau):
        assert lib.sgp_peer_schedule(h, k, ctypes.addressof(out), ctypes.addressof(inp), ctypes.byref(wt)) == 0
        if k % tau:
            assert set(out) == {-1} and set(inp) == {-1} and wt.value == 1.0
        else:
            ref_out, ref_in, ref_w = binding.sgp_schedule(n, peers, k // tau)
            assert list(out) == [v for row in ref_out for v in row]
            assert list(inp) == [v for row in ref_in for v in row]
            assert wt.value == ref_w
    assert lib.sgp_set_biased(h, 1) == 0 and lib.sgp_set_biased(None, 1) == binding.SGP_ERR_INVALID_ARG
    assert lib.sgp_destroy(h) == 0


def test_region_probe_host_paths(lib):
    """Argument checks of sgp_probe_regions and the cases it answers without touching the device:
    fewer than two granules, or granules too small for the probe problem, are one class."""
    import ctypes
    cls = (ctypes.c_int32 * 8)(*([7] * 8))
    ms = (ctypes.c_float * 8)(*([1.0] * 8))
    st = ctypes.c_int32(5)
    fake = 1 << 20                                   # never dereferenced on these paths
    G = 1 << 30
    f = lib.sgp_probe_regions
    assert f(None, 8 * G, G, 4, cls, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    assert f(fake, 8 * G, G, 4, None, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    assert f(fake, 8 * G, G + 1, 4, cls, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    assert f(fake, G // 2, G, 4, cls, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    assert f(fake, 8 * G, G, 0, cls, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    assert f(fake + 4, 8 * G, G, 4, cls, ms, ctypes.byref(st), None) == binding.SGP_ERR_INVALID_ARG
    # eight granules of 1 GiB: the probe problem (four arrays of 512 MiB) does not fit one granule
    assert f(fake, 8 * G, G, 4, cls, ms, ctypes.byref(st), None) == binding.SGP_OK
    assert list(cls) == [0] * 8 and list(ms) == [0.0] * 8 and st.value == 0
    # a single granule
    cls[0] = 7
    assert f(fake, 8 * G, 8 * G, 4, cls, None, ctypes.byref(st), None) == binding.SGP_OK
    assert cls[0] == 0 and st.value == 0
    assert lib.sgp_smooth_region_classes(None, 0) == binding.SGP_OK
    assert lib.sgp_smooth_region_classes(None, 3) == binding.SGP_ERR_INVALID_ARG
