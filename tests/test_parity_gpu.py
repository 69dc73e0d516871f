"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by
element on the same seeded inputs.

Bar.  The float32 oracle rounds every operation separately in the same order the library
specifies, so x, u, w and z are required to be IDENTICAL (which implies the 1e-6 relative bound
of the target; +0 and -0 compare equal).  Against the float64 oracle the bound is the rounding
error of the 6-8 float32 operations per element, stated per test.  Peer indices: bit-exact
(tests/test_host_abi.py).  Statistics: 1e-5 relative against the float64 oracle.
"""
import numpy as np
import pytest
import torch

from oracle import sgp_oracle as O
import paper_1811_10792_amd as sgp
from paper_1811_10792_amd import binding, synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda"
EPS = 2.0 ** -24


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def padded(a, ld, fill=np.float32(7.25)):
    """[n, d] -> device tensor [n, ld] with a sentinel in the padding."""
    n, d = a.shape
    out = np.full((n, ld), fill, np.float32)
    out[:, :d] = a
    return dev(out)


def same(a, b, what):
    if not np.array_equal(a, b):
        bad = np.flatnonzero(a.ravel() != b.ravel())
        denom = np.maximum(np.abs(b.ravel()[bad]), 1e-30)
        rel = np.abs(a.ravel()[bad].astype(np.float64) - b.ravel()[bad]) / denom
        raise AssertionError("%s: %d of %d elements differ, max rel err %.3e (first at %d: %r vs %r)" % (
            what, bad.size, a.size, rel.max(), bad[0], a.ravel()[bad[0]], b.ravel()[bad[0]]))


def random_state(n, d, seed, w_spread=False):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    u = rng.standard_normal((n, d)).astype(np.float32)
    g = rng.standard_normal((n, d)).astype(np.float32)
    w = (0.5 + rng.random(n)).astype(np.float32) if w_spread else np.ones(n, np.float32)
    return x, w, u, g


def run_both(n, d, ld, peers, delay, iters, gamma, mom, seed, k0=0, w_spread=False, zout=True,
             offset=0):
    """Runs `iters` iterations on both sides with fresh random gradients; compares every step."""
    x, w, u, g = random_state(n, d, seed, w_spread)
    rng = np.random.default_rng(seed + 1)
    nest = mom != 0.0
    eng = sgp.SGP(n, d, ld, peers=peers, delay=delay)
    # `offset` floats of slack in front make the base pointers 4-byte but not 16-byte aligned
    def alloc(a):
        flat = torch.full((n * ld + offset,), 7.25, dtype=torch.float32, device=DEV)
        view = flat[offset:].view(n, ld)
        view[:, :d] = dev(a)
        return view
    X, U, G, Z = alloc(x), alloc(u), alloc(g), alloc(np.zeros_like(x))
    W = dev(w)
    st = O.Delay1State(n, d, np.float32) if delay else None
    xo, wo, uo = x.copy(), w.copy(), u.copy()
    for it in range(iters):
        k = k0 + it
        g = rng.standard_normal((n, d)).astype(np.float32)
        G[:, :d] = dev(g)
        eng.step(X, W, U if nest else None, G, Z if zout else None, gamma, mom, k)
        if not zout:
            eng.debias(X, W, Z)
        P = O.mixing_matrix(n, peers, k, np.float32)
        if delay:
            zo = O.step_delay1(P, xo, wo, uo if nest else None, g, gamma, mom, st, nesterov=nest)
        else:
            zo = O.step(P, xo, wo, uo if nest else None, g, gamma, mom, nesterov=nest)
        tag = "n=%d d=%d ld=%d peers=%d delay=%d k=%d" % (n, d, ld, peers, delay, k)
        same(host(X)[:, :d], xo, "x " + tag)
        same(host(W), wo, "w " + tag)
        same(host(Z)[:, :d], zo, "z " + tag)
        if nest:
            same(host(U)[:, :d], uo, "u " + tag)
        else:
            same(host(U)[:, :d], u, "u untouched " + tag)
    for T in (X, U, G, Z):                                   # padding is never written
        assert (host(T)[:, d:] == 7.25).all()
    eng.close()


# ------------------------------------------------------------------- baseline configurations
def _trajectory(wl, iters):
    """Each side follows its own trajectory: g = h*(z - c) + noise from its own z."""
    n, d = wl.n, wl.d
    h, c, x0 = syn.quadratic_problem(n, d, wl.seed, wl.x_std)
    nest = wl.momentum != 0.0
    eng = sgp.SGP(n, d, peers=wl.peers, delay=wl.delay)
    X, W, U = dev(x0), dev(np.ones(n, np.float32)), dev(np.zeros((n, d), np.float32))
    Z, G = torch.empty_like(X), torch.empty_like(X)
    eng.debias(X, W, Z)                                       # z^(0) = x^(0) / w^(0)
    xo, wo, uo = x0.copy(), np.ones(n, np.float32), np.zeros((n, d), np.float32)
    zo = O.debias(xo, wo)
    same(host(Z), zo, "z0")
    x64, w64, u64 = x0.astype(np.float64), np.ones(n), np.zeros((n, d))
    worst64 = 0.0
    dist_hist = []
    for k in range(iters):
        noise = syn.step_noise(n, d, wl.grad_std, wl.seed, k)
        g_gpu = syn.quadratic_gradient(h, c, host(Z), noise)
        g_orc = syn.quadratic_gradient(h, c, zo, noise)
        G.copy_(dev(g_gpu))
        eng.step(X, W, U if nest else None, G, Z, wl.gamma, wl.momentum, k)
        zo = O.step(O.mixing_matrix(n, wl.peers, k, np.float32), xo, wo, uo if nest else None, g_orc,
                    wl.gamma, wl.momentum, nesterov=nest)
        same(host(Z), zo, "%s z k=%d" % (wl.name, k))
        same(host(X), xo, "%s x k=%d" % (wl.name, k))
        # float64 oracle fed with the SAME float32 gradients and the float32 state of step k
        z64 = O.step(O.mixing_matrix(n, wl.peers, k, np.float64), x64, w64, u64 if nest else None,
                     g_orc.astype(np.float64), wl.gamma, wl.momentum, nesterov=nest)
        scale = np.abs(x64).max() + wl.gamma * 4 * (np.abs(g_orc).max() + np.abs(u64).max())
        worst64 = max(worst64, np.abs(zo - z64).max() / scale)
        x64[:], u64[:] = xo, uo                                # re-synchronise: one-step error only
        if k % 20 == 0 or k == iters - 1:
            dist_hist.append(eng.consensus_stats(Z, W).dist_max)
    assert worst64 <= 16 * EPS, worst64
    eng.close()
    return host(Z), h, c, dist_hist


def test_config1_n4_d1024_sgd_200_iterations():
    wl = syn.WORKLOADS["c1_n4_d1k"]
    z, h, c, dist = _trajectory(wl, wl.iterations)
    # trend: the node average approaches the minimiser of the mean quadratic up to noise and
    # step-size effects, and the nodes stay close to each other
    xstar = syn.quadratic_minimiser(h, c)
    start = np.sqrt(((syn.quadratic_problem(wl.n, wl.d, wl.seed)[2].mean(0) - xstar) ** 2).mean())
    end = np.sqrt(((z.mean(0) - xstar) ** 2).mean())
    assert end < 0.1 * start
    assert dist[-1] < dist[0]


def test_config2_n8_d1m_nesterov_100_iterations():
    wl = syn.WORKLOADS["c2_n8_d1m"]
    _trajectory(wl, wl.iterations)


# ------------------------------------------------------------------- shapes, tails, paths
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 31, 32, 33, 100])
def test_one_peer_all_node_counts(n):
    L = max(1, (n - 1).bit_length())
    run_both(n, 1028, 1028, 1, 0, L + 2, 0.1, 0.9, seed=n, w_spread=True)


@pytest.mark.parametrize("d,ld,offset", [(1, 1, 0), (3, 4, 0), (4, 4, 0), (5, 8, 0), (1023, 1024, 0),
                                         (1025, 1028, 0), (2049, 2051, 0), (4096, 4096, 1),
                                         (70001, 70004, 0), (262147, 262148, 0)])
def test_ragged_sizes_padding_and_alignment(d, ld, offset):
    run_both(8, d, ld, 1, 0, 4, 0.05, 0.9, seed=d, w_spread=True, offset=offset)
    run_both(5, d, ld, 2, 0, 3, 0.05, 0.9, seed=d + 1, w_spread=True, offset=offset)
    run_both(6, d, ld, 2, 1, 4, 0.05, 0.9, seed=d + 2, offset=offset)


@pytest.mark.parametrize("mom,zout", [(0.0, True), (0.0, False), (0.9, False), (0.5, True)])
def test_variants_without_momentum_or_z(mom, zout):
    run_both(8, 3000, 3000, 1, 0, 4, 0.1, mom, seed=3, w_spread=True, zout=zout)
    run_both(8, 3000, 3000, 2, 0, 4, 0.1, mom, seed=4, w_spread=True, zout=zout)
    run_both(8, 3000, 3000, 2, 1, 4, 0.1, mom, seed=5, zout=zout)


@pytest.mark.parametrize("n,peers", [(2, 2), (3, 2), (4, 2), (8, 2), (16, 2), (32, 2), (64, 2), (65, 2),
                                     (100, 3), (16, 3), (16, 4), (256, 2)])
def test_multi_peer_gather(n, peers):
    L = max(1, (n - 1).bit_length())
    run_both(n, 520, 520, peers, 0, min(L + 1, 5), 0.1, 0.9, seed=n + peers, w_spread=True)


@pytest.mark.parametrize("peers,delay", [(1, 0), (1, 1), (2, 1)])
def test_largest_node_count(peers, delay):
    """n = SGP_MAX_NODES: every block forms 1024 weights (16 per work-item of a single-wave block)."""
    run_both(1024, 24, 24, peers, delay, 3, 0.1, 0.9, seed=peers + delay, w_spread=True, k0=9)


@pytest.mark.parametrize("n,d", [(150, 132), (151, 132), (600, 36)])
def test_multi_peer_gather_at_the_node_limits(n, d):
    """The private LDS columns of the gather kernel: 128-bit accesses up to n = 150, scalar ones up
    to n = 600 (more than 64 KiB of LDS per block from n = 64 / n = 255 on)."""
    run_both(n, d, d, 2, 0, 3, 0.1, 0.9, seed=n, w_spread=True)


def test_multi_peer_gather_beyond_the_node_limit_leaves_the_state_untouched():
    n, d = binding.SGP_MAX_NODES_GATHER + 1, 8
    eng = sgp.SGP(n, d, peers=2)
    x, w, u, g = (dev(a) for a in random_state(n, d, 0))
    keep = [t.clone() for t in (x, w, u)]
    z = torch.full_like(x, 5.0)
    with pytest.raises(sgp.SgpError) as e:
        eng.step(x, w, u, g, z, 0.1, 0.9, 0)
    assert e.value.status == binding.SGP_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    for t, t0 in zip((x, w, u), keep):
        assert torch.equal(t, t0)
    assert bool((z == 5.0).all())
    eng.close()


@pytest.mark.parametrize("n,peers", [(1, 1), (2, 1), (4, 1), (16, 1), (32, 1), (5, 2), (16, 2), (33, 2),
                                     (16, 3), (12, 4)])
def test_one_iteration_delay(n, peers):
    L = max(1, (n - 1).bit_length())
    run_both(n, 1540, 1540, peers, 1, L + 3, 0.01, 0.9, seed=n * 7 + peers, k0=0)
    run_both(n, 516, 516, peers, 1, 3, 0.01, 0.0, seed=n * 7 + peers + 1, k0=5)   # may start at any k


def test_delay_sequence_and_reset():
    n, d = 4, 64
    eng = sgp.SGP(n, d, peers=1, delay=1)
    x, w, u, g = (dev(a) for a in random_state(n, d, 0))
    eng.step(x, w, u, g, None, 0.1, 0.9, 3)
    with pytest.raises(sgp.SgpError) as e:
        eng.step(x, w, u, g, None, 0.1, 0.9, 5)              # 4 expected
    assert e.value.status == -4
    eng.step(x, w, u, g, None, 0.1, 0.9, 4)
    eng.reset()
    eng.step(x, w, u, g, None, 0.1, 0.9, 0)
    eng.close()


def test_repeated_runs_are_bitwise_identical():
    n, d = 16, 50000
    x, w, u, g = random_state(n, d, 9)
    outs = []
    for _ in range(3):
        eng = sgp.SGP(n, d)
        X, W, U, G = dev(x), dev(w), dev(u), dev(g)
        Z = torch.empty_like(X)
        for k in range(5):
            eng.step(X, W, U, G, Z, 0.1, 0.9, k)
        s = eng.consensus_stats(Z, W, per_node=True)
        outs.append((host(X), host(Z), host(U), s.per_node, s.dist_max))
        eng.close()
    for o in outs[1:]:
        assert all(np.array_equal(a, b) for a, b in zip(o[:3], outs[0][:3]))
        assert o[3] == outs[0][3] and o[4] == outs[0][4]


# ------------------------------------------------------------------- statistics
@pytest.mark.parametrize("n,d,ld", [(1, 100, 100), (2, 7, 8), (4, 1024, 1024), (8, 4099, 4100),
                                    (32, 300001, 300004), (33, 5000, 5000), (100, 2050, 2052),
                                    (16, 1 << 20, 1 << 20)])
def test_consensus_stats(n, d, ld):
    rng = np.random.default_rng(n * 1000 + d)
    base = rng.standard_normal(d).astype(np.float32)
    for spread in (1.0, 1e-4):                                # nodes far apart / near consensus
        z = (base[None, :] + spread * rng.standard_normal((n, d))).astype(np.float32)
        w = (0.5 + rng.random(n)).astype(np.float32)
        eng = sgp.SGP(n, d, ld)
        s = eng.consensus_stats(padded(z, ld, fill=np.float32(1e6)), dev(w), per_node=True)
        dist, ref = O.consensus_stats(z, w)
        tol = 1e-5
        if n > 1:
            assert np.abs(np.array(s.per_node) - dist).max() <= tol * dist.max()
            assert abs(s.dist_max - ref["max"]) <= tol * ref["max"]
            assert abs(s.dist_mean - ref["mean"]) <= tol * ref["mean"]
            assert abs(s.dist_min - ref["min"]) <= tol * ref["min"]
            assert s.argmax == int(np.argmax(dist)) and s.argmin == int(np.argmin(dist))
        else:
            assert s.dist_max == 0.0 and s.dist_min == 0.0
        assert abs(s.w_sum - ref["w_sum"]) <= 1e-12 * ref["w_sum"]
        assert abs(s.zbar_norm - ref["zbar_norm"]) <= tol * ref["zbar_norm"]
        eng.close()


def test_stats_exact_consensus_is_zero():
    n, d = 32, 10000
    z = np.tile(np.random.default_rng(0).standard_normal(d).astype(np.float32), (n, 1))
    eng = sgp.SGP(n, d)
    s = eng.consensus_stats(dev(z), dev(np.ones(n, np.float32)))
    assert s.dist_max == 0.0 and s.dist_mean == 0.0 and s.w_sum == n
    eng.close()


def test_exact_averaging_on_device():
    # gamma = 0, n = 32: after 5 iterations every node holds the average (sums of halves are
    # exact here because the inputs are small integers)
    n, d = 32, 4096
    x = np.random.default_rng(1).integers(-64, 64, (n, d)).astype(np.float32)
    eng = sgp.SGP(n, d)
    X, W, G = dev(x), dev(np.ones(n, np.float32)), dev(np.zeros((n, d), np.float32))
    Z = torch.empty_like(X)
    for k in range(2, 7):
        eng.step(X, W, None, G, Z, 0.0, 0.0, k)
    assert np.array_equal(host(Z), np.tile(x.mean(0, dtype=np.float64).astype(np.float32), (n, 1)))
    assert eng.consensus_stats(Z, W).dist_max == 0.0
    eng.close()


# ------------------------------------------------------------------- full-size spot checks
_ALLOC = None


@pytest.fixture(scope="module", autouse=True)
def _release_the_arena_after_this_module():
    """The arena holds nearly all device memory: whatever runs after this module gets it back."""
    yield
    global _ALLOC
    _ALLOC = None
    if torch.cuda.is_available():
        torch.cuda.empty_cache()


def _bench_allocator():
    """The benchmark's region-aware allocator, set up once for the full-size tests."""
    global _ALLOC
    if _ALLOC is None:
        from paper_1811_10792_amd.placement import StateAllocator
        torch.cuda.empty_cache()
        _ALLOC = StateAllocator("regions")
    return _ALLOC


def test_placement_probe_finds_regions_and_separates_the_written_streams():
    alloc = _bench_allocator()
    info = alloc.describe()
    assert info["mode"] == "regions"
    t = {r: alloc.floats(r, 4, 1 << 20) for r in ("x", "u", "z", "g")}
    info = alloc.describe()
    classes = len(set(info["region_of_granule"]))
    if info["structured"]:                       # the written streams go to different regions
        assert len({info["arrays"][r] for r in ("x", "u", "z")}) == min(3, classes)
    ptrs = sorted((v.data_ptr(), v.numel() * 4) for v in t.values())
    assert all(a + n <= b for (a, n), (b, _) in zip(ptrs, ptrs[1:]))     # disjoint
    assert all(p % 4096 == 0 for p, _ in ptrs)
    alloc.reset()


def _full_size_spot_check(wl, steps, count=3000, force_stats=False):
    """Model-sized state generated on the device, the launch configuration the benchmark times;
    the oracle recomputes a sample of coordinates (coordinates are independent, so a column
    slice of the oracle is exact), including the first tile and the ragged tail."""
    n, d = wl.n, wl.d
    ld = syn.padded_ld(d)                                      # the benchmark's row stride
    alloc = _bench_allocator()                                 # and its placement of the arrays
    X = syn.device_normal(n, ld, wl.x_std, wl.seed, 3, out=alloc.floats("x", n, ld))
    U = syn.device_normal(n, ld, wl.grad_std, wl.seed, 6,     # a non-trivial momentum buffer
                          out=alloc.floats("u", n, ld))
    W = torch.ones(n, dtype=torch.float32, device=DEV)
    Z = alloc.floats("z", n, ld)
    Gbuf = alloc.floats("g", n, ld)
    # also around the places where the launch moves from one XCD's share of the blocks to the next
    # (256 coordinates per block in the one-peer, gather and complete kernels, 2048 in the overlap
    # kernels) and where a row crosses a 2 GiB multiple of the array
    around = syn.partition_boundaries(d, ld, n, 2048 if wl.delay else 256)
    cols = syn.sample_columns(d, count, wl.seed, around=around, halo=512 if wl.delay else 128)
    cidx = torch.from_numpy(cols).to(DEV)
    xo, uo = host(X[:, cidx]), host(U[:, cidx])
    wo = np.ones(n, np.float32)
    complete = wl.topology == "complete"
    adam = wl.optimizer == "adam"
    eng = sgp.SGP(n, d, ld, topology=1 if complete else 0, peers=wl.peers, delay=wl.delay)
    if wl.delay:
        eng.set_message_buffers(alloc.floats("msg0", n, ld), alloc.floats("msg1", n, ld))
    st = O.OsgpState(n, len(cols), np.float32, wl.delay) if wl.delay else None
    V2 = alloc.floats("v", n, ld).zero_() if adam else None
    vo = np.zeros_like(xo) if adam else None
    pad0 = [host(T[:, d:]).copy() for T in (X, U)]
    s_fused = None
    for k in range(steps):
        G = syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + k, out=Gbuf)
        g = host(G[:, cidx])
        if adam:
            eng.step_adam(X, W, U, V2, G, Z, wl.gamma, 0.9, 0.98, 1e-8, k + 1, k)
        elif wl.stats_each_step or force_stats:                # what the benchmark calls
            s_fused = eng.step_stats(X, W, U, G, Z, wl.gamma, wl.momentum, k, per_node=True)
        else:
            eng.step(X, W, U, G, Z, wl.gamma, wl.momentum, k)
        if complete:
            P = np.full((n, n), np.float32(1.0) / np.float32(n), dtype=np.float32)
        else:
            P = O.mixing_matrix(n, wl.peers, k // max(1, wl.delay), np.float32)
        kw = dict(nesterov=False, adam=O.adam_params(0.9, 0.98, 1e-8, k + 1, np.float32), v=vo) if adam else {}
        if wl.delay:
            zo = O.step_osgp(P, xo, wo, uo, g, wl.gamma, wl.momentum, st, k, **kw)
        else:
            zo = O.step(P, xo, wo, uo, g, wl.gamma, wl.momentum, **kw)
        if adam:
            same(host(V2[:, cidx]), vo, "%s second moment k=%d" % (wl.name, k))
        same(host(X[:, cidx]), xo, "%s x k=%d" % (wl.name, k))
        same(host(Z[:, cidx]), zo, "%s z k=%d" % (wl.name, k))
        same(host(U[:, cidx]), uo, "%s u k=%d" % (wl.name, k))
        same(host(W), wo, "%s w k=%d" % (wl.name, k))
    if force_stats and not wl.stats_each_step:
        # too large for the host oracle in reasonable time: the fused kernel's statistics against
        # the stand-alone pass over the z it wrote (itself checked against the oracle at the sizes
        # the host can handle), and against the oracle on the first 2^20 coordinates
        assert eng.last_step_kernel().endswith("_stats")
        s_full = eng.consensus_stats(Z, W, per_node=True)
        assert np.abs(np.array(s_fused.per_node) - np.array(s_full.per_node)).max() <= 1e-5 * s_full.dist_max
        assert abs(s_fused.zbar_norm - s_full.zbar_norm) <= 1e-5 * s_full.zbar_norm
        assert s_fused.w_sum == s_full.w_sum and s_fused.argmax == s_full.argmax
        dsl = 1 << 20
        sl = sgp.SGP(n, dsl, ld)
        s = sl.consensus_stats(Z, W, per_node=True)
        dist, ref = O.consensus_stats(host(Z[:, :dsl]), wo)
        assert np.abs(np.array(s.per_node) - dist).max() <= 1e-5 * dist.max()
        sl.close()
    if wl.stats_each_step:
        # the statistics the fused kernel returned with the last step, against the oracle on the
        # whole z it wrote (a few seconds of host time), and the stand-alone pass on the same z
        zh = np.ascontiguousarray(host(Z)[:, :d])
        dist, ref = O.consensus_stats(zh, wo)
        del zh
        s_full = eng.consensus_stats(Z, W, per_node=True)
        for sres in (s_fused, s_full):
            assert np.abs(np.array(sres.per_node) - dist).max() <= 1e-5 * ref["max"]
            assert abs(sres.dist_max - ref["max"]) <= 1e-5 * ref["max"]
            assert abs(sres.dist_mean - ref["mean"]) <= 1e-5 * ref["mean"]
            assert abs(sres.dist_min - ref["min"]) <= 1e-5 * ref["min"]
            assert abs(sres.zbar_norm - ref["zbar_norm"]) <= 1e-5 * ref["zbar_norm"]
            assert sres.argmax == int(np.argmax(dist)) and sres.w_sum == n
        dsl = 1 << 20
        sl = sgp.SGP(n, dsl, ld)
        s = sl.consensus_stats(Z, W, per_node=True)           # first 2^20 coordinates, stride ld
        dist, ref = O.consensus_stats(host(Z[:, :dsl]), wo)
        assert np.abs(np.array(s.per_node) - dist).max() <= 1e-5 * dist.max()
        assert abs(s.dist_max - ref["max"]) <= 1e-5 * ref["max"]
        sl.close()
    for T, p0 in zip((X, U), pad0):                            # padding columns stay untouched
        assert np.array_equal(host(T[:, d:]), p0)
    eng.close()
    del X, U, Z, G, Gbuf
    alloc.reset()


def _full_size_every_element(wl, steps, k0=0):
    """Consecutive iterations at full size in the benchmark's launch configuration and placement,
    EVERY element of x, u, z (and w) compared with the float32 oracle after every iteration (the
    oracle steps the whole state on the host: a few seconds per iteration)."""
    n, d = wl.n, wl.d
    ld = syn.padded_ld(d)
    alloc = _bench_allocator()
    X = syn.device_normal(n, ld, wl.x_std, wl.seed, 3, out=alloc.floats("x", n, ld))
    U = syn.device_normal(n, ld, wl.grad_std, wl.seed, 6, out=alloc.floats("u", n, ld))
    W = torch.ones(n, dtype=torch.float32, device=DEV)
    Z = alloc.floats("z", n, ld)
    Gbuf = alloc.floats("g", n, ld)

    def whole(T):                                    # the d used columns of every row, on the host
        return np.ascontiguousarray(T[:, :d].cpu().numpy())
    xo, uo, wo = whole(X), whole(U), np.ones(n, np.float32)
    eng = sgp.SGP(n, d, ld, peers=wl.peers, delay=0)
    for k in range(k0, k0 + steps):
        G = syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + k, out=Gbuf)
        g = whole(G)
        if wl.stats_each_step:                       # the benchmark's call
            s_fused = eng.step_stats(X, W, U, G, Z, wl.gamma, wl.momentum, k, per_node=True)
        else:
            eng.step(X, W, U, G, Z, wl.gamma, wl.momentum, k)
        zo = O.step(O.mixing_matrix(n, wl.peers, k, np.float32), xo, wo, uo, g, wl.gamma, wl.momentum)
        del g
        for T, ref, what in ((X, xo, "x"), (U, uo, "u"), (Z, zo, "z")):
            for i in range(n):                       # row by row: bounded host memory
                got = T[i, :d].cpu().numpy()
                if not np.array_equal(got, ref[i]):
                    bad = np.flatnonzero(got != ref[i])
                    raise AssertionError("%s %s k=%d node %d: %d elements differ, first at coordinate %d"
                                         % (wl.name, what, k, i, bad.size, bad[0]))
        same(host(W), wo, "%s w k=%d" % (wl.name, k))
        if wl.stats_each_step and k == k0 + steps - 1:
            dist, ref = O.consensus_stats(zo, wo)
            assert np.abs(np.array(s_fused.per_node) - dist).max() <= 1e-5 * ref["max"]
            assert abs(s_fused.zbar_norm - ref["zbar_norm"]) <= 1e-5 * ref["zbar_norm"]
        del zo
    eng.close()
    del X, U, Z, G, Gbuf
    alloc.reset()


def test_full_size_config4_every_element_over_all_five_hops():
    _full_size_every_element(syn.WORKLOADS["c4_n32_resnet50"], steps=5, k0=3)


def test_full_size_config3_every_element_over_all_four_hops():
    _full_size_every_element(syn.WORKLOADS["c3_n16_resnet50"], steps=4)


def test_full_size_two_peer_blocking():
    _full_size_spot_check(syn.WORKLOADS["x4_n32_resnet50_2peer"], steps=3)
    _full_size_spot_check(syn.WORKLOADS["x5_n16_resnet50_2peer"], steps=2)


def test_full_size_config3_n16_resnet50():
    _full_size_spot_check(syn.WORKLOADS["c3_n16_resnet50"], steps=2)


def test_full_size_config4_n32_resnet50():
    _full_size_spot_check(syn.WORKLOADS["c4_n32_resnet50"], steps=3)


def test_full_size_config4_whole_run_of_50_iterations():
    _full_size_spot_check(syn.WORKLOADS["c4_n32_resnet50"], steps=50, count=600)


def test_full_size_config5_n16_transformer_two_peer_overlap():
    _full_size_spot_check(syn.WORKLOADS["c5_n16_transformer_2peer_overlap"], steps=3)


def test_full_size_config5_with_fused_statistics():
    _full_size_spot_check(syn.WORKLOADS["c5_n16_transformer_2peer_overlap"], steps=3, force_stats=True)


def test_full_size_two_peer_blocking_with_fused_statistics():
    _full_size_spot_check(syn.WORKLOADS["x4_n32_resnet50_2peer"], steps=2, force_stats=True)


def test_full_size_transformer_two_peer_tau2():
    _full_size_spot_check(syn.WORKLOADS["x1_n16_transformer_2peer_tau2"], steps=5)


def test_full_size_resnet50_complete_graph():
    _full_size_spot_check(syn.WORKLOADS["x2_n32_resnet50_complete"], steps=2)


def test_full_size_transformer_two_peer_overlap_adam():
    _full_size_spot_check(syn.WORKLOADS["x3_n16_transformer_2peer_overlap_adam"], steps=3)
