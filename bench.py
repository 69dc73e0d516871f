#!/usr/bin/env python3
"""Benchmark of the SGP update on one MI355X.

A "step" is one pass of the whole hot path over all n simulated nodes: peer schedule, momentum
update, local step, PushSum mix of x and w, de-bias and (for the workloads that ask for it) the
consensus statistics: statistics accumulated inside the step kernel, reduced and copied to the
host in every step, and picked up by the host one step late so that the stream never drains
(sgp_step_stats_begin / _end; --sync-stats: picked up before the next step is launched,
sgp_step_stats; --separate-stats: one sgp_step call plus one sgp_consensus_stats call).  All state and a
small rotating pool of pre-drawn gradient buffers are resident in HBM before the timed region;
drawing gradients is not part of the step (g is an input of the method).

Prints ONE JSON line: node-parameter updates per second (n*d*K / wall time of the K steps, a timed
region that holds the steps and nothing else), the roofline of the dominant kernel (the step
kernel, timed in a second pass of the same steps with HIP events on the stream it runs on) with the
whole-step fraction beside it, the same steps with ordinary allocations instead of the region-aware
placement, and the CPU oracle timed at the workload's full size where the host can hold it (with
all cores) and on a slice (with one core).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def algorithmic_bytes_per_update(wl) -> float:
    """HBM bytes the method itself must move per node-parameter: state read once, state written
    once (the gather costs nothing when a work-item owns a coordinate for all nodes)."""
    nest = wl.momentum != 0.0
    adam = wl.optimizer == "adam"
    moments = 2 if adam else 1 if nest else 0
    reads = 4 * (2 + moments)                     # x, g, (u), (second moment)
    writes = 4 * (2 + moments)                    # x, z, (u), (second moment)
    total = float(reads + writes)
    if wl.delay:                                  # previous messages read, new messages written,
        total += 8.0 / wl.delay                   # at one iteration in every tau
    if wl.storage != "f32":                       # storage experiment: g and z held as bfloat16,
        total -= 4.0                              # 2 bytes less for each
        if wl.storage == "bf16_guz":              # and the momentum: 2 less read, 2 less written
            total -= 4.0
    return total


def read_traffic(workload_name, kernel, n, d, ld):
    """HBM bytes per launch of the step kernel as hardware counters measured them, read from the
    committed summary of an EARLIER profiling run (profiles/step_kernel_<workload>_pmc.txt): counters
    cannot be collected inside a timing run.  Returned with its source only when the summary names
    the kernel and the shape that this run launched; otherwise (None, None)."""
    rel = os.path.join("profiles", "step_kernel_%s_pmc.txt" % workload_name)
    try:
        text = open(os.path.join(ROOT, rel)).read()
    except OSError:
        return None, None

    def field(name):
        m = re.search(r"^%s:\s*(\S+)" % name, text, re.M)
        return m.group(1) if m else None
    if (field("kernel") != kernel or field("n") != str(n) or field("d") != str(d) or field("ld") != str(ld)
            or field("traffic_bytes_per_launch") is None):
        return None, None
    return float(field("traffic_bytes_per_launch")), rel


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


FULL_D_LIMIT_BYTES = 16 << 30     # the oracle leg runs at full d when one state array set fits this


def _oracle_run(wl, dcols, threads, max_steps, budget_s):
    """Times `max_steps` oracle iterations (or as many as fit the budget, at least one) of workload
    wl restricted to its first `dcols` coordinates (coordinates are independent, so that is exact)."""
    import numpy as np
    from oracle import sgp_oracle as O
    from paper_1811_10792_amd import synthetic as syn
    O.set_threads(threads)
    n = wl.n
    blk = min(dcols, 1 << 21)                       # drawn once, repeated along the row: the values
    reps = (dcols + blk - 1) // blk                 # do not change what the oracle computes per element
    x = np.ascontiguousarray(np.tile(syn.normal((n, blk), wl.x_std, wl.seed, 3), (1, reps))[:, :dcols])
    g = np.ascontiguousarray(np.tile(syn.normal((n, blk), wl.grad_std, wl.seed, 4, 0), (1, reps))[:, :dcols])
    u = np.zeros((n, dcols), np.float32)
    w = np.ones(n, np.float32)
    st = O.OsgpState(n, dcols, np.float32, wl.delay) if wl.delay else None
    nest = wl.momentum != 0.0
    adam = wl.optimizer == "adam"
    v = np.zeros((n, dcols), np.float32) if adam else None
    steps, t0 = 0, time.perf_counter()
    while True:
        if wl.topology == "complete":
            P = np.full((n, n), np.float32(1.0) / np.float32(n), dtype=np.float32)
        else:
            P = O.mixing_matrix(n, wl.peers, steps // max(1, wl.delay), np.float32)
        ad = O.adam_params(0.9, 0.98, 1e-8, steps + 1, np.float32) if adam else None
        if wl.delay:
            z = O.step_osgp(P, x, w, u if (nest or adam) else None, g, wl.gamma, wl.momentum, st, steps,
                            nesterov=nest, adam=ad, v=v)
        else:
            z = O.step(P, x, w, u if (nest or adam) else None, g, wl.gamma, wl.momentum, nesterov=nest,
                       adam=ad, v=v)
        if wl.stats_each_step:
            O.consensus_stats(z, w)
        del z
        steps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or steps >= max_steps:
            break
    return n * dcols * steps / el, steps, el


def cpu_baseline(wl):
    """The oracle as it stands (float32 variant, dense P per coordinate, plus the float64
    statistics when the workload reports them) timed on the host: with all cores at the workload's
    full size when the state fits the host comfortably (every configuration but the Transformer-sized
    ones, which run on a slice of 2^21 coordinates per node), and with one core on a slice."""
    from oracle import sgp_oracle as O
    cores = len(os.sched_getaffinity(0))
    threads = max(1, min(cores, O.max_threads()))
    arrays = 5 if wl.optimizer == "adam" else 4
    full = wl.n * wl.d * 4 * arrays <= FULL_D_LIMIT_BYTES
    dcols = wl.d if full else min(wl.d, 1 << 21)
    value, steps, el = _oracle_run(wl, dcols, threads, max_steps=3 if dcols > (1 << 22) else 50, budget_s=12.0)
    d1 = min(wl.d, 1 << 19)
    v1, s1, e1 = _oracle_run(wl, d1, 1, max_steps=3 if wl.n * d1 > (1 << 22) else 50, budget_s=6.0)
    what = ("all %d coordinates per node" % wl.d) if full else \
        ("a contiguous slice of %d of its %d coordinates per node" % (dcols, wl.d))
    return {"value": value, "unit": "node-param updates/s", "cores": threads, "kind": "oracle",
            "sample": "%d steps of %s on %s, all %d nodes, %.1f s" % (steps, wl.name, what, wl.n, el),
            "single_core": {"value": v1, "cores": 1,
                            "sample": "%d steps on a contiguous slice of %d coordinates per node, %.1f s" % (s1, d1, e1)},
            "cpu_model": cpu_model()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4_n32_resnet50")
    ap.add_argument("--pool", type=int, default=2, help="pre-drawn gradient buffers to rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stats", action="store_true", help="skip the per-step consensus statistics")
    ap.add_argument("--stats", action="store_true",
                    help="take the consensus statistics in every step also for a workload that does not ask for them")
    ap.add_argument("--sync-stats", action="store_true",
                    help="fetch the statistics of every step before launching the next one (sgp_step_stats) "
                         "instead of one step late (sgp_step_stats_begin / _end)")
    ap.add_argument("--separate-stats", action="store_true",
                    help="run sgp_step and sgp_consensus_stats as two calls instead of sgp_step_stats")
    ap.add_argument("--graph", action="store_true",
                    help="capture one cycle of the peer schedule (L iterations) into a HIP graph and time "
                         "replays of it: for small models, where launch overhead dominates (blocking mode "
                         "without statistics only; the step kernels are not timed individually)")
    ap.add_argument("--placement", choices=("regions", "default"), default="regions",
                    help="regions: carve the state arrays out of one arena so that the written "
                         "streams x, u, z sit in different HBM regions (found by timing); "
                         "default: plain allocations")
    ap.add_argument("--no-default-placement", action="store_true",
                    help="skip the extra leg that repeats the steps with ordinary allocations")
    ap.add_argument("--strict-placement", action="store_true",
                    help="exit non-zero when the region-aware placement was asked for but is degraded")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain copy kernel over one state array (a transfer of "
                         "known size, against which hardware traffic counters are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all simulated nodes live in one HBM); "
                 "--gpus %d is not supported" % args.gpus)

    import torch
    import paper_1811_10792_amd as sgp
    from paper_1811_10792_amd import synthetic as syn
    from paper_1811_10792_amd.placement import StateAllocator

    wl = syn.WORKLOADS[args.workload]
    n, d = wl.n, wl.d
    torch.cuda.set_device(0)
    nest = wl.momentum != 0.0
    ld = syn.padded_ld(d)                 # rows start on 1 KiB boundaries
    alloc = StateAllocator(args.placement)
    complete = wl.topology == "complete"
    eng = sgp.SGP(n, d, ld, topology=1 if complete else 0, peers=wl.peers, delay=wl.delay)
    X = syn.device_normal(n, ld, wl.x_std, wl.seed, 3, out=alloc.floats("x", n, ld))
    W = torch.ones(n, dtype=torch.float32, device="cuda")
    adam = wl.optimizer == "adam"
    V2 = alloc.floats("v", n, ld).zero_() if adam else None
    h16 = wl.storage != "f32"                     # storage experiment: some arrays held as bfloat16
    storage = {"f32": 0, "bf16_gz": sgp.binding.SGP_STORE_BF16_GZ,
               "bf16_guz": sgp.binding.SGP_STORE_BF16_GZ | sgp.binding.SGP_STORE_BF16_U}[wl.storage]

    def halves(role, name=None):                  # [n, ld] bfloat16 carved like a float array of half the width
        return alloc.floats(role, n, ld // 2, name).view(torch.bfloat16)
    if wl.storage == "bf16_guz":
        U = halves("u").zero_()
    else:
        U = alloc.floats("u", n, ld).zero_()
    Z = halves("z") if h16 else alloc.floats("z", n, ld)
    pool = []
    for i in range(max(1, args.pool)):
        if h16:
            G = halves("g", "g%d" % i)
            G.copy_(syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + i))
        else:
            G = syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + i, out=alloc.floats("g", n, ld, "g%d" % i))
        pool.append(G)
    if wl.delay:
        eng.set_message_buffers(alloc.floats("msg0", n, ld), alloc.floats("msg1", n, ld))
    do_stats = (wl.stats_each_step or args.stats) and not args.no_stats and not h16
    stream = torch.cuda.current_stream()

    k = 0
    last = None

    pipelined = do_stats and not args.separate_stats and not args.sync_stats and wl.optimizer != "adam"

    pending = [0]           # statistics enqueued and not yet fetched

    def drain():
        r = None
        while pending[0]:
            r = eng.step_stats_end()
            pending[0] -= 1
        return r

    def one_step(k):
        if pipelined:       # enqueue step k, then pick up the statistics of step k-1
            eng.step_stats_begin(X, W, U if nest else None, pool[k % len(pool)], Z, wl.gamma, wl.momentum, k)
            pending[0] += 1
            if pending[0] < 2:
                return None
            pending[0] -= 1
            return eng.step_stats_end()
        if adam:
            eng.step_adam(X, W, U, V2, pool[k % len(pool)], Z, wl.gamma, 0.9, 0.98, 1e-8, k + 1, k)
            return eng.consensus_stats(Z, W) if do_stats else None
        if h16:
            eng.step_bf16(X, W, U, pool[k % len(pool)], Z, wl.gamma, wl.momentum, k, storage)
            return None
        if do_stats and not args.separate_stats:    # one call: statistics fused into the step kernel
            return eng.step_stats(X, W, U if nest else None, pool[k % len(pool)], Z, wl.gamma,
                                  wl.momentum, k)
        eng.step(X, W, U if nest else None, pool[k % len(pool)], Z, wl.gamma, wl.momentum, k)
        return eng.consensus_stats(Z, W) if do_stats else None

    if args.graph:
        if do_stats or wl.delay or adam:
            sys.exit("bench.py --graph: blocking workloads without statistics only")
        L = max(1, (n - 1).bit_length())
        one_step(0)                                   # sets up the library's device tables
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for kk in range(L):
                one_step(kk)
        reps = max(1, args.steps // L)
        for _ in range(max(1, args.warmup // L)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        steps = reps * L
        print(json.dumps({
            "metric": "SGP node-param updates/sec (n*d/step time) + achieved HBM GB/s vs peak",
            "value": n * d * steps / elapsed, "unit": "node-param updates/s", "n_gpus": 1, "steps": steps,
            "warmup": args.warmup, "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": wl.name, "n": n, "d": d, "ld": ld, "launch": "HIP graph of %d iterations" % L},
            "roofline": {"bound": "hbm", "kernel": "whole graph",
                         "achieved": algorithmic_bytes_per_update(wl) * n * d * steps / elapsed / 1e9,
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": algorithmic_bytes_per_update(wl) * n * d * steps / elapsed / 1e9 / HBM_PEAK_GBPS,
                         "traffic": None}}), flush=True)
        eng.close()
        return

    for _ in range(args.warmup):
        last = one_step(k)
        k += 1
    if args.calibrate_copy:
        sgp.sgp_copy(X, X.clone() if h16 else pool[0]) if h16 else sgp.sgp_copy(Z, pool[0])   # n*ld*4 bytes read and written
    torch.cuda.synchronize()

    # ---- the timed region: exactly --steps steps, nothing but the steps ------------------------
    t0 = time.perf_counter()
    for i in range(args.steps):
        last = one_step(k)
        k += 1
    if pipelined:
        last = drain()                    # the last step's statistics, inside the timed region
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_name = eng.last_step_kernel()  # what the library launched, as it reports it

    # ---- a second pass of the same steps for the roofline of the dominant kernel: HIP events
    # around the step kernel, recorded by the library on the stream it launches on (kept out of the
    # timed region above, where the two extra event records per step would be part of the step)
    eng.set_kernel_timing(True)
    kern_ms = []
    ksteps = min(args.steps, 60)
    for i in range(ksteps):
        one_step(k)
        k += 1
        if i % 32 == 31:
            kern_ms += eng.step_kernel_times()
    drain()
    torch.cuda.synchronize()
    kern_ms += eng.step_kernel_times()
    eng.set_kernel_timing(False)
    assert len(kern_ms) == ksteps, (len(kern_ms), ksteps)
    avg_kern_s = sum(kern_ms) / len(kern_ms) / 1e3
    bpu = algorithmic_bytes_per_update(wl)
    achieved = bpu * n * d / avg_kern_s / 1e9
    whole = bpu * n * d * args.steps / elapsed / 1e9
    traffic, traffic_source = read_traffic(wl.name, kernel_name, n, d, ld)
    placement = alloc.describe()
    degraded = args.placement == "regions" and not (placement["mode"] == "regions" and placement.get("structured"))
    out = {
        "metric": "SGP node-param updates/sec (n*d/step time) + achieved HBM GB/s vs peak",
        "value": n * d * args.steps / elapsed,
        "unit": "node-param updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not h16 else "f32 arithmetic, bfloat16 storage of %s" % ("g, z, u" if wl.storage == "bf16_guz" else "g, z"),
        "data": "synthetic",
        "config": {"workload": wl.name, "n": n, "d": d, "ld": ld, "topology": wl.topology,
                   "peers": wl.peers, "delay": wl.delay,
                   "optimizer": wl.optimizer, "momentum": wl.momentum, "gamma": wl.gamma,
                   "consensus_stats_each_step": bool(do_stats),
                   "stats_fetch": ("one step late" if pipelined else "every step") if do_stats else None,
                   "gradient_pool": len(pool),
                   "placement": placement},
        # True: the region-aware placement was asked for but the arena could not be had or its probe
        # found no region structure, so the arrays sit wherever the allocator put them
        "placement_degraded": bool(degraded),
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_update": bpu,
                     "kernel_ms_avg": avg_kern_s * 1e3, "kernel_ms_median": sorted(kern_ms)[len(kern_ms) // 2],
                     "kernel_ms_min": min(kern_ms), "kernel_timing": "separate pass of %d steps" % ksteps,
                     # the whole step as the timed region saw it (every launch, gap and copy included)
                     "whole_step_achieved": whole, "whole_step_frac": whole / HBM_PEAK_GBPS},
    }
    if last is not None:
        out["consensus_dist_max_last"] = last.dist_max
    # context, not a target: the paper reports end-to-end training results only
    out["paper_reported"] = {"comparable": False,
                             "what": "ImageNet/ResNet-50, 90 epochs, one DGX-1 (8 V100) per node, 10 Gbps Ethernet: "
                                     "1-peer SGP 16 / 32 nodes 75.9 % in 3.2 h / 75.0 % in 1.7 h; AllReduce SGD "
                                     "76.3 % in 8.5 h / 76.2 % in 5.1 h; no per-iteration update throughput is published"}
    eng.close()
    del X, U, Z, V2, pool, alloc, G      # every view into the arena, so that it is really released
    torch.cuda.empty_cache()
    if args.placement == "regions" and not args.no_default_placement and not h16:
        out["default_placement"] = default_placement_leg(wl, ld, args, bpu)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)
    if degraded and args.strict_placement:
        sys.exit("bench.py: region-aware placement was requested but is degraded (see placement_degraded)")


def default_placement_leg(wl, ld, args, bpu):
    """The same steps with ordinary back-to-back allocations (what a caller gets who hands the
    library whatever the allocator returned), reported beside the region-aware figure."""
    import torch
    import paper_1811_10792_amd as sgp
    from paper_1811_10792_amd import synthetic as syn
    n, d = wl.n, wl.d
    nest = wl.momentum != 0.0
    adam = wl.optimizer == "adam"
    eng = sgp.SGP(n, d, ld, topology=1 if wl.topology == "complete" else 0, peers=wl.peers, delay=wl.delay)
    X = syn.device_normal(n, ld, wl.x_std, wl.seed, 3)
    U = torch.zeros((n, ld), dtype=torch.float32, device="cuda")
    V2 = torch.zeros((n, ld), dtype=torch.float32, device="cuda") if adam else None
    W = torch.ones(n, dtype=torch.float32, device="cuda")
    Z = torch.empty((n, ld), dtype=torch.float32, device="cuda")
    pool = [syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + i) for i in range(max(1, args.pool))]
    do_stats = wl.stats_each_step and not args.no_stats
    pipelined = do_stats and not adam

    def one_step(k):
        G = pool[k % len(pool)]
        if pipelined:
            eng.step_stats_begin(X, W, U if nest else None, G, Z, wl.gamma, wl.momentum, k)
            if k > 0:
                eng.step_stats_end()
        elif adam:
            eng.step_adam(X, W, U, V2, G, Z, wl.gamma, 0.9, 0.98, 1e-8, k + 1, k)
        else:
            eng.step(X, W, U if nest else None, G, Z, wl.gamma, wl.momentum, k)
    k = 0
    for _ in range(max(2, args.warmup)):
        one_step(k)
        k += 1
    torch.cuda.synchronize()
    steps = max(1, min(args.steps, 20))
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(k)
        k += 1
    if pipelined:
        eng.step_stats_end()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    eng.close()
    whole = bpu * n * d * steps / el / 1e9
    return {"ms_per_step": el / steps * 1e3, "steps": steps, "value": n * d * steps / el,
            "whole_step_frac": whole / HBM_PEAK_GBPS}


if __name__ == "__main__":
    main()
