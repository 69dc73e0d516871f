"""Seeded synthetic workloads for the SGP step (no SGP arithmetic lives here).

These stand in for the paper's ImageNet/ResNet-50 and WMT'16/Transformer runs, which only matter
to the update path through their shapes: the node counts 4..32 of the scaling experiments and
model-sized flat parameter vectors.  Both the GPU tests/benchmark and the CPU-oracle tests draw
their inputs from this module so that the two sides see identical bits.

Conventions: every array is float32, shape [n, d] (one row per simulated node); "N(0, s)" uses
s as the standard deviation; a per-node quadratic f_i(x) = 0.5 * sum_e h_i[e] (x[e] - c_i[e])^2
has gradient h_i * (z - c_i), to which per-step noise is added.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n: int                 # simulated nodes
    d: int                 # parameters per node
    peers: int             # out-peers per iteration on the directed exponential graph
    delay: int             # tau: 0 = blocking SGP, 1 = messages arrive one iteration late, ...
    gamma: float
    momentum: float        # 0 -> plain SGD step (Alg. 1), else Nesterov (Alg. 3)
    iterations: int
    gradient: str          # "quadratic" (depends on z) or "fresh" (drawn anew per step)
    grad_std: float        # noise std ("quadratic") or gradient std ("fresh")
    x_std: float           # std of the initial x
    stats_each_step: bool = False
    seed: int = 0
    optimizer: str = "nesterov"   # "nesterov" (momentum 0: plain SGD) or "adam" (beta 0.9 / 0.98, eps 1e-8)
    topology: str = "exp"  # "exp": directed exponential graph; "complete": every entry of P is 1/n
    storage: str = "f32"   # "f32", or the 16-bit storage experiment: "bf16_gz" (g and z held as
                           # bfloat16) / "bf16_guz" (the momentum as well); arithmetic is float32 always


# The five configurations of the build's baseline description, in its order, then extensions.
WORKLOADS = {
    "c1_n4_d1k": Workload("c1_n4_d1k", 4, 1024, 1, 0, 0.1, 0.0, 200, "quadratic", 0.01, 1.0),
    "c2_n8_d1m": Workload("c2_n8_d1m", 8, 1 << 20, 1, 0, 0.05, 0.9, 100, "quadratic", 0.1, 1.0),
    "c3_n16_resnet50": Workload("c3_n16_resnet50", 16, 25_557_032, 1, 0, 0.1, 0.9, 50, "fresh",
                                1e-3, 0.05),
    "c4_n32_resnet50": Workload("c4_n32_resnet50", 32, 25_557_032, 1, 0, 0.1, 0.9, 50, "fresh",
                                1e-3, 0.05, stats_each_step=True),
    "c5_n16_transformer_2peer_overlap": Workload("c5_n16_transformer_2peer_overlap", 16,
                                                 213_000_000, 2, 1, 1e-3, 0.9, 20, "fresh",
                                                 1e-4, 0.05),
    # beyond the baseline description: configuration 5 with tau = 2 (communication every second
    # iteration, messages two iterations late)
    "x1_n16_transformer_2peer_tau2": Workload("x1_n16_transformer_2peer_tau2", 16, 213_000_000, 2, 2,
                                              1e-3, 0.9, 20, "fresh", 1e-4, 0.05),
    # configuration 4's shape on the complete graph (the AllReduce-equivalent end of the hybrid schemes)
    "x2_n32_resnet50_complete": Workload("x2_n32_resnet50_complete", 32, 25_557_032, 1, 0, 0.1, 0.9, 50,
                                         "fresh", 1e-3, 0.05, topology="complete"),
    # configuration 5 with Adam as the local optimiser (what the paper's Transformer runs use)
    "x3_n16_transformer_2peer_overlap_adam": Workload("x3_n16_transformer_2peer_overlap_adam", 16,
                                                      213_000_000, 2, 1, 1e-3, 0.0, 20, "fresh", 1e-4, 0.05,
                                                      optimizer="adam"),
    # the two-peer blocking runs of the paper's communication-topology comparison (16 and 32 nodes,
    # ResNet-50-sized vectors): configuration 3's / 4's shape with two out-peers and no delay
    "x4_n32_resnet50_2peer": Workload("x4_n32_resnet50_2peer", 32, 25_557_032, 2, 0, 0.1, 0.9, 50, "fresh",
                                      1e-3, 0.05),
    "x5_n16_resnet50_2peer": Workload("x5_n16_resnet50_2peer", 16, 25_557_032, 2, 0, 0.1, 0.9, 50, "fresh",
                                      1e-3, 0.05),
    # a node count that is not a power of two (the exponential graph is then regular but a cycle of
    # the schedule no longer averages exactly), with the statistics taken every step
    "x6_n24_resnet50_stats": Workload("x6_n24_resnet50_stats", 24, 25_557_032, 1, 0, 0.1, 0.9, 50, "fresh",
                                      1e-3, 0.05, stats_each_step=True),
    # the paper's 1-peer overlap runs on ResNet-50 (one out-peer, one iteration of delay) on
    # configuration 4's shape, with the statistics taken every step
    "x7_n32_resnet50_overlap_stats": Workload("x7_n32_resnet50_overlap_stats", 32, 25_557_032, 1, 1, 0.1, 0.9, 50,
                                              "fresh", 1e-3, 0.05, stats_each_step=True),
    # storage experiment, not in the paper: configuration 4's shape (without the statistics) with g
    # and z, then also the momentum, held in memory as bfloat16; 20 and 16 bytes per node-parameter
    "h1_n32_resnet50_bf16_gz": Workload("h1_n32_resnet50_bf16_gz", 32, 25_557_032, 1, 0, 0.1, 0.9, 50, "fresh",
                                        1e-3, 0.05, storage="bf16_gz"),
    "h2_n32_resnet50_bf16_guz": Workload("h2_n32_resnet50_bf16_guz", 32, 25_557_032, 1, 0, 0.1, 0.9, 50, "fresh",
                                         1e-3, 0.05, storage="bf16_guz"),
}


def padded_ld(d: int, multiple: int = 256) -> int:
    """Row stride used by the benchmark and the full-size tests: d rounded up to a multiple of 256
    elements, so that every node's row starts on a 1 KiB boundary."""
    return (d + multiple - 1) // multiple * multiple


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), *[int(s) for s in stream]])


def normal(shape, std: float, seed: int, *stream: int) -> np.ndarray:
    """float32 N(0, std) array; (seed, *stream) names the draw."""
    return (_rng(seed, *stream).standard_normal(shape, dtype=np.float32) * np.float32(std))


def uniform(shape, lo: float, hi: float, seed: int, *stream: int) -> np.ndarray:
    r = _rng(seed, *stream).random(shape, dtype=np.float32)
    return (np.float32(lo) + r * np.float32(hi - lo)).astype(np.float32)


def quadratic_problem(n: int, d: int, seed: int = 0, x_std: float = 1.0):
    """Curvatures h ~ U[0.5, 2], centres c ~ N(0, 1) and the initial x ~ N(0, x_std)."""
    h = uniform((n, d), 0.5, 2.0, seed, 1)
    c = normal((n, d), 1.0, seed, 2)
    x0 = normal((n, d), x_std, seed, 3)
    return h, c, x0


def step_noise(n: int, d: int, std: float, seed: int, k: int) -> np.ndarray:
    """Noise (or, for the "fresh" workloads, the whole gradient) of iteration k."""
    return normal((n, d), std, seed, 4, k)


def quadratic_gradient(h: np.ndarray, c: np.ndarray, z: np.ndarray, noise: np.ndarray) -> np.ndarray:
    """g_i = h_i * (z_i - c_i) + noise_i, each operation rounded to float32."""
    t = (z - c).astype(np.float32)
    t = (h * t).astype(np.float32)
    return (t + noise).astype(np.float32)


def quadratic_minimiser(h: np.ndarray, c: np.ndarray) -> np.ndarray:
    """argmin of (1/n) sum_i f_i: x*[e] = sum_i h_i[e] c_i[e] / sum_i h_i[e] (float64)."""
    h64 = h.astype(np.float64)
    return (h64 * c.astype(np.float64)).sum(0) / h64.sum(0)


def initial_state(wl: Workload):
    """x^(0), w^(0) = 1, u^(0) = 0 on the host."""
    x0 = normal((wl.n, wl.d), wl.x_std, wl.seed, 3)
    return x0, np.ones((wl.n,), np.float32), np.zeros((wl.n, wl.d), np.float32)


# ---- device-side generators for the model-sized workloads (torch used for memory only) -------

def device_normal(n: int, ld: int, std: float, seed: int, stream: int, device="cuda", out=None):
    """float32 [n, ld] N(0, std) tensor drawn on the device from a seeded generator (padding
    columns, if ld exceeds d, are drawn too; the library never touches them).  With `out`, the
    draw goes into that tensor (same values as a fresh one: the generator only sees the count)."""
    import torch
    if out is None:
        out = torch.empty((n, ld), dtype=torch.float32, device=device)
    gen = torch.Generator(device=out.device)
    gen.manual_seed((int(seed) * 1_000_003 + int(stream)) & 0x7FFFFFFFFFFFFFFF)
    out.normal_(0.0, float(std), generator=gen)
    return out


def sample_columns(d: int, count: int, seed: int = 0, tile: int = 1024, around=(), halo: int = 512) -> np.ndarray:
    """Sorted, distinct coordinate indices for spot checks at full size: the first and last
    `tile` coordinates (first tile and ragged tail of any launch), `count` random ones, and the
    `halo` coordinates before and after every coordinate listed in `around` (places where a
    launch's work partition or the address arithmetic changes regime)."""
    parts = [np.arange(0, min(tile, d)), np.arange(max(0, d - tile), d),
             _rng(seed, 5).integers(0, d, size=count)]
    for c in around:
        parts.append(np.arange(max(0, int(c) - halo), min(d, int(c) + halo)))
    return np.unique(np.concatenate(parts)).astype(np.int64)


def partition_boundaries(d: int, ld: int, n: int, coords_per_block: int, parts: int = 8,
                         byte_period: int = 1 << 31) -> list:
    """Coordinates at which a launch over d coordinates in blocks of `coords_per_block` switches
    from one of `parts` contiguous shares of the blocks to the next, and coordinates at which some
    row of an [n, ld] float32 array crosses a multiple of `byte_period` bytes from the array's
    start.  Pure index arithmetic, used to pick spot-check columns."""
    G = (d + coords_per_block - 1) // coords_per_block
    q, r = divmod(G, parts)
    out = [(x * q + min(x, r)) * coords_per_block for x in range(1, parts)]
    per = byte_period // 4
    for i in range(n):
        first = -(-(i * ld) // per) * per            # first multiple of the period at or after the row's start
        for e in range(first, i * ld + d, per):
            out.append(e - i * ld)
    return sorted({c for c in out if 0 < c < d})
