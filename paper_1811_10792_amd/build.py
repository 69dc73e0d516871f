"""Builds the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libsgp_hip.so")
OBJ_DIR = os.path.join(PKG, "_build")

# translation units as (source, object name, defines), the slowest to compile first.  The walk with
# fused statistics is compiled once per variant of its kernel (see the head of sgp_walk_stats.hip).
def _walk(nest: int, cached: int, msg: int):
    return ("sgp_walk_stats.hip", "sgp_walk_stats_n%dc%dm%d" % (nest, cached, msg),
            ["-DSGP_WALK_NEST=%d" % nest, "-DSGP_WALK_CACHED=%d" % cached, "-DSGP_WALK_MSG=%d" % msg])


UNITS = [
    _walk(1, 0, 2), _walk(0, 0, 2), _walk(1, 0, 1), _walk(0, 0, 1), _walk(1, 0, 0), _walk(1, 1, 0), _walk(0, 0, 0),
    _walk(0, 1, 0),
    ("sgp.hip", "sgp", []),
    ("sgp_overlap.hip", "sgp_overlap", []),
    ("sgp_gather.hip", "sgp_gather", ["-DSGP_GATHER_STATS=0"]),
    ("sgp_gather.hip", "sgp_gather_stats", ["-DSGP_GATHER_STATS=1"]),
]

HIPCC_FLAGS = [
    "-O3", "-std=c++20", "--offload-arch=gfx950", "-fPIC",
    # every float operation rounds on its own: the results are specified operation by operation
    "-ffp-contract=off",
    # no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _quiet(text: str) -> str:
    return "\n".join(l for l in text.splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), proc.stdout))
    out = _quiet(proc.stdout)
    if verbose and out.strip():
        print(out, flush=True)


def build(verbose: bool = False, extra_flags=(), jobs: int | None = None) -> str:
    """Compiles every translation unit (side by side, `jobs` at a time) and links the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if jobs is None:
        jobs = max(1, min(len(UNITS), os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))
    tag = ".%d" % os.getpid()
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, name + tag + ".o") for _, name, _ in UNITS]
    tmp = LIB + ".tmp" + tag
    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            futs = [pool.submit(_run, [hipcc, *HIPCC_FLAGS, *defs, *extra_flags, "-I", INCLUDE, "-c",
                                       os.path.join(CSRC, src), "-o", o], verbose)
                    for (src, _, defs), o in zip(UNITS, objs)]
            for f in futs:
                f.result()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, LIB)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
