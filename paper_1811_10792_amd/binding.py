"""Thin ctypes binding of the C ABI in include/sgp.h: argument marshalling only.

PyTorch appears here for device memory and streams (tensor.data_ptr(), the current stream's
handle); every arithmetic step runs in the HIP library.  There is no fallback: if the library has
not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsgp_hip.so")

SGP_OK = 0
SGP_ERR_INVALID_ARG = -1
SGP_ERR_UNSUPPORTED = -2
SGP_ERR_ALIGNMENT = -3
SGP_ERR_SEQUENCE = -4
SGP_ERR_HIP = -5
SGP_ERR_NOMEM = -6
SGP_TOPO_DIRECTED_EXP = 0
SGP_TOPO_COMPLETE = 1
SGP_TOPO_CUSTOM = 2
SGP_MAX_NODES_GATHER = 600
SGP_STORE_BF16_GZ = 1
SGP_STORE_BF16_U = 2

# every symbol include/sgp.h declares
EXPORTS = ("sgp_create", "sgp_destroy", "sgp_reset", "sgp_step", "sgp_debias",
           "sgp_consensus_stats", "sgp_peer_schedule", "sgp_schedule", "sgp_status_string",
           "sgp_last_hip_error", "sgp_copy", "sgp_set_kernel_timing", "sgp_step_kernel_times",
           "sgp_set_message_buffers", "sgp_step_stats", "sgp_set_biased", "sgp_set_topology",
           "sgp_set_mixing", "sgp_set_weight_decay", "sgp_step_adam",
           "sgp_pregossip_stats", "sgp_step_stats_begin", "sgp_step_stats_end",
           "sgp_consensus_stats_noalloc", "sgp_last_step_kernel", "sgp_probe_regions",
           "sgp_smooth_region_classes", "sgp_step_bf16", "sgp_debug_fail_alloc",
           "sgp_placer_create", "sgp_placer_destroy", "sgp_placer_reset", "sgp_placer_take",
           "sgp_stream_pattern")


class SgpError(RuntimeError):
    def __init__(self, status: int, name: str, where: str):
        super().__init__("%s failed: %s (%d)" % (where, name, status))
        self.status = status


class _CStats(ctypes.Structure):
    _fields_ = [("dist_max", ctypes.c_double), ("dist_mean", ctypes.c_double),
                ("dist_min", ctypes.c_double), ("w_sum", ctypes.c_double),
                ("zbar_norm", ctypes.c_double), ("argmax", ctypes.c_int32),
                ("argmin", ctypes.c_int32)]


@dataclass
class Stats:
    dist_max: float
    dist_mean: float
    dist_min: float
    w_sum: float
    zbar_norm: float
    argmax: int
    argmin: int
    per_node: Optional[list] = None


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libsgp_hip.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "HIP library %s is missing: build it first (python -m paper_1811_10792_amd.build); "
            "there is no CPU fallback" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.sgp_create.argtypes = [ctypes.POINTER(vp), i32, i64, i64, i32, i32, i32]
    lib.sgp_destroy.argtypes = [vp]
    lib.sgp_reset.argtypes = [vp]
    lib.sgp_step.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, i64, vp]
    lib.sgp_step_adam.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, f32, i64, i64, vp]
    lib.sgp_debias.argtypes = [vp, vp, vp, vp, vp]
    lib.sgp_consensus_stats.argtypes = [vp, vp, vp, ctypes.POINTER(_CStats), vp, vp]
    lib.sgp_pregossip_stats.argtypes = [vp, vp, vp, vp, vp, f32, f32, ctypes.POINTER(_CStats), vp, vp]
    lib.sgp_peer_schedule.argtypes = [vp, i64, vp, vp, ctypes.POINTER(f32)]
    lib.sgp_schedule.argtypes = [i32, i32, i64, vp, vp, ctypes.POINTER(f32)]
    lib.sgp_status_string.argtypes = [ctypes.c_int]
    lib.sgp_status_string.restype = ctypes.c_char_p
    lib.sgp_last_hip_error.argtypes = [vp]
    lib.sgp_copy.argtypes = [vp, vp, i64, vp]
    lib.sgp_stream_pattern.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(vp), i32, i64, vp]
    lib.sgp_set_message_buffers.argtypes = [vp, vp, vp]
    lib.sgp_step_stats.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, i64, ctypes.POINTER(_CStats), vp, vp]
    lib.sgp_set_biased.argtypes = [vp, ctypes.c_int]
    lib.sgp_set_weight_decay.argtypes = [vp, f32, ctypes.c_int]
    lib.sgp_set_topology.argtypes = [vp, i32, i32]
    lib.sgp_set_mixing.argtypes = [vp, vp, vp, i32]
    lib.sgp_step_stats_begin.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, i64, vp]
    lib.sgp_step_stats_end.argtypes = [vp, ctypes.POINTER(_CStats), vp]
    lib.sgp_set_kernel_timing.argtypes = [vp, ctypes.c_int]
    lib.sgp_consensus_stats_noalloc.argtypes = [i32, i64, i64, vp, vp, vp, vp]
    lib.sgp_step_kernel_times.argtypes = [vp, vp, i32, ctypes.POINTER(i32)]
    lib.sgp_probe_regions.argtypes = [vp, i64, i64, i32, vp, vp, ctypes.POINTER(i32), vp]
    lib.sgp_smooth_region_classes.argtypes = [vp, i32]
    lib.sgp_debug_fail_alloc.argtypes = [i32]
    lib.sgp_placer_create.argtypes = [ctypes.POINTER(vp), vp, i32, i64]
    lib.sgp_placer_destroy.argtypes = [vp]
    lib.sgp_placer_reset.argtypes = [vp]
    lib.sgp_placer_take.argtypes = [vp, i32, i64, ctypes.POINTER(i64), ctypes.POINTER(i32)]
    lib.sgp_step_bf16.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, i64, i32, vp]
    lib.sgp_last_step_kernel.argtypes = [vp]
    lib.sgp_last_step_kernel.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("sgp_status_string", "sgp_last_step_kernel"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().sgp_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != SGP_OK:
        raise SgpError(status, status_string(status), where)


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or None)."""
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream; None -> torch's current stream."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def sgp_schedule(n: int, peers: int, k: int):
    """Handle-free peer schedule: (out_peers[n][peers], in_peers[n][peers], weight)."""
    lib = load_library()
    out = (ctypes.c_int32 * (n * peers))()
    inp = (ctypes.c_int32 * (n * peers))()
    wt = ctypes.c_float()
    _check(lib.sgp_schedule(n, peers, k, ctypes.addressof(out), ctypes.addressof(inp),
                            ctypes.byref(wt)), "sgp_schedule")
    rows = lambda a: [list(a[i * peers:(i + 1) * peers]) for i in range(n)]
    return rows(out), rows(inp), wt.value


def sgp_copy(dst, src, nbytes: Optional[int] = None, stream=None) -> None:
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    _check(load_library().sgp_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "sgp_copy")


def sgp_stream_pattern(reads, writes, nbytes: Optional[int] = None, stream=None) -> None:
    """One launch of the structure-free stream kernel: reads every tensor of `reads`, writes every
    tensor of `writes` (see include/sgp.h); all of the same size."""
    both = list(reads) + list(writes)
    if nbytes is None:
        nbytes = both[0].numel() * both[0].element_size() if both else 0
    r = (ctypes.c_void_p * max(1, len(reads)))(*[_ptr(t) for t in reads])
    w = (ctypes.c_void_p * max(1, len(writes)))(*[_ptr(t) for t in writes])
    _check(load_library().sgp_stream_pattern(r, len(reads), w, len(writes), nbytes, _stream(stream)),
           "sgp_stream_pattern")


def sgp_consensus_stats_noalloc(n: int, d: int, ld: int, z, w, out_device, stream=None) -> None:
    """Statistics of z into the device tensor out_device ([8 + n] float64) without any allocation
    and without synchronising; layout as in include/sgp.h."""
    _check(load_library().sgp_consensus_stats_noalloc(n, d, ld, _ptr(z), _ptr(w), _ptr(out_device),
                                                      _stream(stream)), "sgp_consensus_stats_noalloc")


def sgp_probe_regions(arena_ptr: int, arena_bytes: int, granule_bytes: int, max_classes: int = 4, stream=None):
    """Classifies the granules of a device arena by mutual interference (see include/sgp.h).
    Returns (classes, first_pass_ms, structured)."""
    count = max(1, arena_bytes // granule_bytes)
    cls = (ctypes.c_int32 * count)()
    ms = (ctypes.c_float * count)()
    structured = ctypes.c_int32()
    _check(load_library().sgp_probe_regions(arena_ptr, arena_bytes, granule_bytes, max_classes,
                                            ctypes.addressof(cls), ctypes.addressof(ms),
                                            ctypes.byref(structured), _stream(stream)), "sgp_probe_regions")
    return list(cls), list(ms), bool(structured.value)


def sgp_smooth_region_classes(classes):
    """Host-only clean-up of raw region classes (outlier granules, renumbering); returns a new list."""
    buf = (ctypes.c_int32 * max(1, len(classes)))(*[int(c) for c in classes])
    _check(load_library().sgp_smooth_region_classes(ctypes.addressof(buf), len(classes)),
           "sgp_smooth_region_classes")
    return list(buf[:len(classes)])


ROLES = {"x": 0, "g": 1, "u": 2, "z": 3, "msg0": 4, "msg1": 5, "v": 6}


class RegionPlacer:
    """Owner of one sgp_placer: hands out byte offsets into a probed arena (host-only)."""

    def __init__(self, classes, granule_bytes: int):
        self._lib = load_library()
        self._p = ctypes.c_void_p()
        buf = (ctypes.c_int32 * max(1, len(classes)))(*[int(c) for c in classes])
        _check(self._lib.sgp_placer_create(ctypes.byref(self._p), ctypes.addressof(buf), len(classes),
                                           granule_bytes), "sgp_placer_create")

    def take(self, role: str, nbytes: int):
        """(offset, region class) of a fresh range for an array in the given role; MemoryError when
        nothing fits."""
        off, cls = ctypes.c_int64(), ctypes.c_int32()
        rc = self._lib.sgp_placer_take(self._p, ROLES[role], nbytes, ctypes.byref(off), ctypes.byref(cls))
        if rc == SGP_ERR_NOMEM:
            raise MemoryError("arena exhausted")
        _check(rc, "sgp_placer_take")
        return off.value, cls.value

    def reset(self) -> None:
        _check(self._lib.sgp_placer_reset(self._p), "sgp_placer_reset")

    def close(self) -> None:
        if getattr(self, "_p", None) is not None and self._p.value:
            self._lib.sgp_placer_destroy(self._p)
            self._p = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SGP:
    """Owner of one sgp_handle.  Tensors are float32 CUDA tensors of shape [n, ld] / [n]."""

    def __init__(self, n: int, d: int, ld: Optional[int] = None, topology: int = SGP_TOPO_DIRECTED_EXP,
                 peers: int = 1, delay: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.n, self.d, self.ld = n, d, d if ld is None else ld
        self.peers, self.delay = peers, delay
        _check(self._lib.sgp_create(ctypes.byref(self._h), n, d, self.ld, topology, peers, delay),
               "sgp_create")

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.sgp_destroy(self._h)
            self._h = ctypes.c_void_p()
        self._msg_keepalive = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _expect(self, t, name, rows_only=False):
        if t is None:
            return
        if not t.is_cuda or t.dtype.is_floating_point is False or t.element_size() != 4 \
                or not t.is_contiguous():
            raise ValueError("%s must be a contiguous float32 CUDA tensor" % name)
        want = self.n if rows_only else self.n * self.ld
        if t.numel() != want:
            raise ValueError("%s has %d elements, expected %d" % (name, t.numel(), want))

    def step(self, x, w, m, g, z_out, gamma: float, momentum: float, k: int, stream=None) -> None:
        for t, name in ((x, "x"), (m, "m"), (g, "g"), (z_out, "z_out")):
            self._expect(t, name)
        self._expect(w, "w", rows_only=True)
        _check(self._lib.sgp_step(self._h, _ptr(x), _ptr(w), _ptr(m), _ptr(g), _ptr(z_out),
                                  gamma, momentum, k, _stream(stream)), "sgp_step")

    def step_adam(self, x, w, m1, m2, g, z_out, gamma: float, beta1: float, beta2: float, eps: float,
                  t: int, k: int, stream=None) -> None:
        """One iteration with Adam as the local optimiser (m1, m2: its two moments, t: its step count)."""
        for tt, name in ((x, "x"), (m1, "m1"), (m2, "m2"), (g, "g"), (z_out, "z_out")):
            self._expect(tt, name)
        self._expect(w, "w", rows_only=True)
        _check(self._lib.sgp_step_adam(self._h, _ptr(x), _ptr(w), _ptr(m1), _ptr(m2), _ptr(g), _ptr(z_out),
                                       gamma, beta1, beta2, eps, t, k, _stream(stream)), "sgp_step_adam")

    def step_bf16(self, x, w, m, g16, z16, gamma: float, momentum: float, k: int, storage: int,
                  stream=None) -> None:
        """Bandwidth experiment: one iteration with g and z (and, with SGP_STORE_BF16_U, m) held as
        bfloat16 tensors of shape [n, ld]; x and w stay float32."""
        import torch
        self._expect(x, "x")
        self._expect(w, "w", rows_only=True)
        for t, name, half in ((g16, "g16", True), (z16, "z16", True), (m, "m", bool(storage & SGP_STORE_BF16_U))):
            want = torch.bfloat16 if half else torch.float32
            if not t.is_cuda or t.dtype != want or not t.is_contiguous() or t.numel() != self.n * self.ld:
                raise ValueError("%s must be a contiguous %s CUDA tensor of %d elements" % (name, want, self.n * self.ld))
        _check(self._lib.sgp_step_bf16(self._h, _ptr(x), _ptr(w), _ptr(m), _ptr(g16), _ptr(z16), gamma, momentum,
                                       k, storage, _stream(stream)), "sgp_step_bf16")

    def step_stats(self, x, w, m, g, z_out, gamma: float, momentum: float, k: int,
                   per_node: bool = False, stream=None) -> Stats:
        """One iteration plus the consensus statistics of the z it wrote (fused where possible)."""
        for t, name in ((x, "x"), (m, "m"), (g, "g"), (z_out, "z_out")):
            self._expect(t, name)
        self._expect(w, "w", rows_only=True)
        cs = _CStats()
        buf = (ctypes.c_double * self.n)() if per_node else None
        _check(self._lib.sgp_step_stats(self._h, _ptr(x), _ptr(w), _ptr(m), _ptr(g), _ptr(z_out),
                                        gamma, momentum, k, ctypes.byref(cs),
                                        ctypes.addressof(buf) if per_node else None,
                                        _stream(stream)), "sgp_step_stats")
        return Stats(cs.dist_max, cs.dist_mean, cs.dist_min, cs.w_sum, cs.zbar_norm, cs.argmax,
                     cs.argmin, list(buf) if per_node else None)

    def step_stats_begin(self, x, w, m, g, z_out, gamma: float, momentum: float, k: int, stream=None) -> None:
        """Enqueues iteration k and the statistics of its z; fetch them later with step_stats_end()."""
        for t, name in ((x, "x"), (m, "m"), (g, "g"), (z_out, "z_out")):
            self._expect(t, name)
        self._expect(w, "w", rows_only=True)
        _check(self._lib.sgp_step_stats_begin(self._h, _ptr(x), _ptr(w), _ptr(m), _ptr(g), _ptr(z_out),
                                              gamma, momentum, k, _stream(stream)), "sgp_step_stats_begin")

    def step_stats_end(self, per_node: bool = False) -> Stats:
        """The oldest result of step_stats_begin not yet fetched (waits for it if necessary)."""
        cs = _CStats()
        buf = (ctypes.c_double * self.n)() if per_node else None
        _check(self._lib.sgp_step_stats_end(self._h, ctypes.byref(cs),
                                            ctypes.addressof(buf) if per_node else None), "sgp_step_stats_end")
        return Stats(cs.dist_max, cs.dist_mean, cs.dist_min, cs.w_sum, cs.zbar_norm, cs.argmax,
                     cs.argmin, list(buf) if per_node else None)

    def debias(self, x, w, z, stream=None) -> None:
        self._expect(x, "x")
        self._expect(z, "z")
        self._expect(w, "w", rows_only=True)
        _check(self._lib.sgp_debias(self._h, _ptr(x), _ptr(w), _ptr(z), _stream(stream)),
               "sgp_debias")

    def consensus_stats(self, z, w, per_node: bool = False, stream=None) -> Stats:
        self._expect(z, "z")
        self._expect(w, "w", rows_only=True)
        cs = _CStats()
        buf = (ctypes.c_double * self.n)() if per_node else None
        _check(self._lib.sgp_consensus_stats(self._h, _ptr(z), _ptr(w), ctypes.byref(cs),
                                             ctypes.addressof(buf) if per_node else None,
                                             _stream(stream)), "sgp_consensus_stats")
        return Stats(cs.dist_max, cs.dist_mean, cs.dist_min, cs.w_sum, cs.zbar_norm, cs.argmax,
                     cs.argmin, list(buf) if per_node else None)

    def pregossip_stats(self, x, w, m, g, gamma: float, momentum: float, per_node: bool = False,
                        stream=None) -> Stats:
        """Statistics of xh / w, the parameters after the local step and before communication."""
        for t, name in ((x, "x"), (m, "m"), (g, "g")):
            self._expect(t, name)
        self._expect(w, "w", rows_only=True)
        cs = _CStats()
        buf = (ctypes.c_double * self.n)() if per_node else None
        _check(self._lib.sgp_pregossip_stats(self._h, _ptr(x), _ptr(w), _ptr(m), _ptr(g), gamma, momentum,
                                             ctypes.byref(cs), ctypes.addressof(buf) if per_node else None,
                                             _stream(stream)), "sgp_pregossip_stats")
        return Stats(cs.dist_max, cs.dist_mean, cs.dist_min, cs.w_sum, cs.zbar_norm, cs.argmax,
                     cs.argmin, list(buf) if per_node else None)

    def peer_schedule(self, k: int):
        n, peers = self.n, self.peers
        out = (ctypes.c_int32 * (n * peers))()
        inp = (ctypes.c_int32 * (n * peers))()
        wt = ctypes.c_float()
        _check(self._lib.sgp_peer_schedule(self._h, k, ctypes.addressof(out), ctypes.addressof(inp),
                                           ctypes.byref(wt)), "sgp_peer_schedule")
        rows = lambda a: [list(a[i * peers:(i + 1) * peers]) for i in range(n)]
        return rows(out), rows(inp), wt.value

    def set_message_buffers(self, buf0, buf1) -> None:
        """Overlap mode: keep the two message buffers in these caller-owned [n, ld] tensors."""
        self._expect(buf0, "buf0")
        self._expect(buf1, "buf1")
        self._msg_keepalive = (buf0, buf1)
        _check(self._lib.sgp_set_message_buffers(self._h, _ptr(buf0), _ptr(buf1)),
               "sgp_set_message_buffers")

    def set_topology(self, topology: int, peers: int = 1) -> None:
        """Switches topology / peer count from the next step on (blocking mode only)."""
        _check(self._lib.sgp_set_topology(self._h, topology, peers), "sgp_set_topology")
        self.peers = peers

    def set_mixing(self, in_idx, in_weight) -> None:
        """SGP_TOPO_CUSTOM: sparse rows of P as [n][entries] lists (index -1 = unused entry)."""
        n = self.n
        entries = len(in_idx[0])
        idx = (ctypes.c_int32 * (n * entries))(*[int(v) for row in in_idx for v in row])
        wts = (ctypes.c_float * (n * entries))(*[float(v) for row in in_weight for v in row])
        _check(self._lib.sgp_set_mixing(self._h, ctypes.addressof(idx), ctypes.addressof(wts), entries),
               "sgp_set_mixing")

    def set_weight_decay(self, weight_decay: float, on_numerator: bool = False) -> None:
        """g + weight_decay * z (or * x with on_numerator) from the next step on."""
        _check(self._lib.sgp_set_weight_decay(self._h, weight_decay, int(on_numerator)),
               "sgp_set_weight_decay")

    def set_biased(self, biased: bool) -> None:
        """Ablation without the push-sum weight: later steps write z = x."""
        _check(self._lib.sgp_set_biased(self._h, int(biased)), "sgp_set_biased")

    def set_kernel_timing(self, enable: bool) -> None:
        _check(self._lib.sgp_set_kernel_timing(self._h, int(enable)), "sgp_set_kernel_timing")

    def step_kernel_times(self):
        """Durations (ms) of the step kernels timed since the last call (at most 64, oldest first);
        waits for the latest one."""
        buf = (ctypes.c_float * 64)()
        cnt = ctypes.c_int32()
        _check(self._lib.sgp_step_kernel_times(self._h, ctypes.addressof(buf), 64, ctypes.byref(cnt)),
               "sgp_step_kernel_times")
        return list(buf[:cnt.value])

    def last_step_kernel(self) -> str:
        """Name of the step kernel the latest successful step launched."""
        return self._lib.sgp_last_step_kernel(self._h).decode()

    def reset(self) -> None:
        _check(self._lib.sgp_reset(self._h), "sgp_reset")

    def last_hip_error(self) -> int:
        return int(self._lib.sgp_last_hip_error(self._h))
