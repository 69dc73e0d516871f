"""ctypes front end of the CPU oracle (oracle/sgp_oracle.c).

TEST INFRASTRUCTURE ONLY.  The product package never imports this module; only tests, the
smoke check and the benchmark's CPU-baseline leg do.  It imports nothing from the product
package either.

All arrays are C-contiguous numpy arrays of shape [n, d] (one row per node) and [n]; the dtype
(float64 or float32) picks the arithmetic the C code runs in.  State arrays are updated in
place, as Alg. 1 / Alg. 3 update x, u and w.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "sgp_oracle.c"), os.path.join(_HERE, "sgp_oracle_impl.inc")]
_SO = os.path.join(_HERE, "libsgp_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every float operation separately
    rounded (no fused multiply-add), which the float32 variant relies on."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        tmp = _SO + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c11",
               "-shared", "-fPIC", "-o", tmp, _SRC[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i32, i64 = ctypes.c_int, ctypes.c_int64
            vp = ctypes.c_void_p
            for sfx, real in (("_f64", ctypes.c_double), ("_f32", ctypes.c_float)):
                f = getattr(lib, "sgpo_mixing_matrix" + sfx)
                f.argtypes = [i32, i32, i64, vp]
                f.restype = None
                f = getattr(lib, "sgpo_step" + sfx)
                f.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, real, real, i32, real, i32, vp, vp]
                f.restype = i32
                f = getattr(lib, "sgpo_step_delay1" + sfx)
                f.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, real, real, i32, vp, vp, vp, i32]
                f.restype = i32
                f = getattr(lib, "sgpo_step_osgp" + sfx)
                f.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, real, real, i32, i32, i64, i32,
                              vp, vp, vp, vp, real, i32, vp, vp]
                f.restype = i32
                f = getattr(lib, "sgpo_debias" + sfx)
                f.argtypes = [i32, i64, vp, vp, vp]
                f.restype = None
            lib.sgpo_step_bf16.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, ctypes.c_float, ctypes.c_float, i32]
            lib.sgpo_step_bf16.restype = i32
            lib.sgpo_float_to_bf16.argtypes = [ctypes.c_float]
            lib.sgpo_float_to_bf16.restype = ctypes.c_uint16
            lib.sgpo_bf16_to_float.argtypes = [ctypes.c_uint16]
            lib.sgpo_bf16_to_float.restype = ctypes.c_float
            lib.sgpo_consensus_stats.argtypes = [i32, i64, vp, vp, vp, vp]
            lib.sgpo_consensus_stats.restype = None
            lib.sgpo_set_threads.argtypes = [i32]
            lib.sgpo_get_max_threads.restype = i32
            _lib = lib
    return _lib


def _sfx(dtype) -> str:
    dtype = np.dtype(dtype)
    if dtype == np.float64:
        return "_f64"
    if dtype == np.float32:
        return "_f32"
    raise TypeError("oracle runs in float64 or float32, got %s" % dtype)


def _chk(a, dtype, shape):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags.c_contiguous \
            or tuple(a.shape) != tuple(shape):
        raise ValueError("expected C-contiguous %s array of shape %s, got %s %s" % (
            dtype, shape, getattr(a, "dtype", None), getattr(a, "shape", None)))
    return a.ctypes.data


def set_threads(t: int) -> None:
    _load().sgpo_set_threads(int(t))


def max_threads() -> int:
    return int(_load().sgpo_get_max_threads())


def mixing_matrix(n: int, peers: int, k: int, dtype=np.float64) -> np.ndarray:
    """Dense P^(k) [n, n] of the directed exponential graph; rows receive, columns send."""
    P = np.empty((n, n), dtype=dtype)
    getattr(_load(), "sgpo_mixing_matrix" + _sfx(dtype))(n, peers, k, P.ctypes.data)
    return P


def adam_params(beta1, beta2, eps, t, dtype):
    """The seven Adam scalars in the working precision: beta1, 1 - beta1, beta2, 1 - beta2 and the
    bias corrections 1 - beta1^t, 1 - beta2^t (formed in double, then rounded), eps."""
    dt = np.dtype(dtype).type
    b1, b2 = dt(beta1), dt(beta2)
    return np.array([b1, dt(1) - b1, b2, dt(1) - b2, dt(1.0 - float(b1) ** t), dt(1.0 - float(b2) ** t),
                     dt(eps)], dtype=dtype)


def step(P, x, w, u, g, gamma, m, nesterov=True, wd=0.0, wd_on_x=False, adam=None, v=None):
    """One SGP iteration with mixing matrix P (Alg. 1 if nesterov is False, else Alg. 3).
    Updates x, w (and u) in place and returns z.  wd: weight decay, g + wd * z (or wd * x).
    adam: array from adam_params() -> Adam is the local step, u and v hold its two moments."""
    dt = x.dtype
    n, d = x.shape
    z = np.empty_like(x)
    if u is None:
        if nesterov or adam is not None:
            raise ValueError("momentum needs the buffer u")
        up = None
    else:
        up = _chk(u, dt, (n, d))
    rc = getattr(_load(), "sgpo_step" + _sfx(dt))(
        n, d, _chk(P, dt, (n, n)), _chk(x, dt, (n, d)), _chk(w, dt, (n,)), up,
        _chk(g, dt, (n, d)), z.ctypes.data, float(gamma), float(m), int(bool(nesterov)),
        float(wd), int(bool(wd_on_x)), None if adam is None else _chk(v, dt, (n, d)),
        None if adam is None else _chk(adam, dt, (7,)))
    if rc != 0:
        raise MemoryError("oracle step failed")
    return z


class Delay1State:
    """What 1-overlap SGP carries from one iteration to the next: the previous half-step
    iterates, the senders' previous weights and the previous mixing matrix."""

    def __init__(self, n, d, dtype):
        self.xh_prev = np.zeros((n, d), dtype=dtype)
        self.w_prev = np.zeros((n,), dtype=dtype)
        self.P_prev = np.zeros((n, n), dtype=dtype)
        self.have_prev = False


def step_delay1(P, x, w, u, g, gamma, m, state: Delay1State, nesterov=True):
    """One iteration of 1-overlap SGP (Alg. 2, tau = 1, messages exactly one iteration late)."""
    dt = x.dtype
    n, d = x.shape
    z = np.empty_like(x)
    up = None if u is None else _chk(u, dt, (n, d))
    if up is None and nesterov:
        raise ValueError("momentum needs the buffer u")
    rc = getattr(_load(), "sgpo_step_delay1" + _sfx(dt))(
        n, d, _chk(P, dt, (n, n)), _chk(x, dt, (n, d)), _chk(w, dt, (n,)), up,
        _chk(g, dt, (n, d)), z.ctypes.data, float(gamma), float(m), int(bool(nesterov)),
        _chk(state.xh_prev, dt, (n, d)), _chk(state.w_prev, dt, (n,)),
        _chk(state.P_prev, dt, (n, n)), int(state.have_prev))
    if rc != 0:
        raise MemoryError("oracle step failed")
    state.have_prev = True
    return z


class OsgpState:
    """The one set of messages that tau-overlap SGP has in flight: what the senders held, the
    matrix they used and the iteration at which the set is received (-1: nothing in flight)."""

    def __init__(self, n, d, dtype, tau: int):
        if tau < 1:
            raise ValueError("tau >= 1 (tau = 0 is plain SGP: use step)")
        self.tau = tau
        self.xh_sent = np.zeros((n, d), dtype=dtype)
        self.w_sent = np.zeros((n,), dtype=dtype)
        self.P_sent = np.zeros((n, n), dtype=dtype)
        self.arrival = np.full((1,), -1, dtype=np.int64)


def step_osgp(P, x, w, u, g, gamma, m, state: OsgpState, k: int, nesterov=True, biased=False,
              wd=0.0, wd_on_x=False, adam=None, v=None):
    """Iteration k of tau-overlap SGP (Alg. 2): sends at k % tau == 0 with matrix P, receives what
    was sent tau iterations ago; biased=True returns z = x (the ablation without push-sum weight)."""
    dt = x.dtype
    n, d = x.shape
    z = np.empty_like(x)
    up = None if u is None else _chk(u, dt, (n, d))
    if up is None and nesterov:
        raise ValueError("momentum needs the buffer u")
    rc = getattr(_load(), "sgpo_step_osgp" + _sfx(dt))(
        n, d, _chk(P, dt, (n, n)), _chk(x, dt, (n, d)), _chk(w, dt, (n,)), up,
        _chk(g, dt, (n, d)), z.ctypes.data, float(gamma), float(m), int(bool(nesterov)),
        int(state.tau), int(k), int(bool(biased)), _chk(state.xh_sent, dt, (n, d)),
        _chk(state.w_sent, dt, (n,)), _chk(state.P_sent, dt, (n, n)), state.arrival.ctypes.data,
        float(wd), int(bool(wd_on_x)), None if adam is None else _chk(v, dt, (n, d)),
        None if adam is None else _chk(adam, dt, (7,)))
    if rc != 0:
        raise RuntimeError("oracle step_osgp failed (%d)" % rc)
    return z


def debias(x, w):
    dt = x.dtype
    n, d = x.shape
    z = np.empty_like(x)
    getattr(_load(), "sgpo_debias" + _sfx(dt))(n, d, _chk(x, dt, (n, d)), _chk(w, dt, (n,)),
                                               z.ctypes.data)
    return z


def consensus_stats(z, w):
    """Returns (dist[n], dict(max, mean, min, w_sum, zbar_norm)) computed in float64 from the
    values of z and w as given (float32 inputs are widened exactly)."""
    z64 = np.ascontiguousarray(z, dtype=np.float64)
    w64 = np.ascontiguousarray(w, dtype=np.float64)
    n, d = z64.shape
    dist = np.empty((n,), dtype=np.float64)
    out = np.empty((5,), dtype=np.float64)
    _load().sgpo_consensus_stats(n, d, z64.ctypes.data, w64.ctypes.data, dist.ctypes.data,
                                 out.ctypes.data)
    return dist, {"max": out[0], "mean": out[1], "min": out[2], "w_sum": out[3],
                  "zbar_norm": out[4]}


def float_to_bf16(f: float) -> int:
    """Bit pattern of the bfloat16 nearest to the binary32 value f (ties to even)."""
    return int(_load().sgpo_float_to_bf16(float(np.float32(f))))


def bf16_to_float(h: int) -> float:
    return float(_load().sgpo_bf16_to_float(int(h)))


def step_bf16(P, x, w, u, g16, gamma, m):
    """Storage experiment: one Nesterov iteration with g16 (uint16 bit patterns of bfloat16) as the
    gradient; u is float32 or uint16 (bfloat16 storage of the momentum).  Updates x, w, u in place and
    returns z as uint16 bit patterns."""
    n, d = x.shape
    z16 = np.empty((n, d), dtype=np.uint16)
    u_is_bf16 = u.dtype == np.uint16
    rc = _load().sgpo_step_bf16(n, d, _chk(P, np.float32, (n, n)), _chk(x, np.float32, (n, d)),
                                _chk(w, np.float32, (n,)), _chk(u, np.uint16 if u_is_bf16 else np.float32, (n, d)),
                                _chk(g16, np.uint16, (n, d)), z16.ctypes.data, float(gamma), float(m), int(u_is_bf16))
    if rc != 0:
        raise MemoryError("oracle step failed")
    return z16
