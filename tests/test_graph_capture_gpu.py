"""The step calls are plain kernel launches on the caller's stream (no allocation after the first
call, no memset), so a caller may capture a run of iterations into a HIP graph and replay it: useful
for small models, where launch overhead dominates.  Every replay is checked against the oracle, with
eager work and synchronisation between replays."""
import numpy as np
import pytest
import torch

from oracle import sgp_oracle as O
import paper_1811_10792_amd as sgp

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("n,d,peers", [(8, 4096, 1), (4, 1024, 1), (8, 1030, 2)])
def test_captured_cycle_of_iterations_replays_correctly(n, d, peers):
    rng = np.random.default_rng(n + d)
    L = max(1, (n - 1).bit_length())                     # one full cycle of the peer schedule
    x = rng.standard_normal((n, d)).astype(np.float32)
    u, w = np.zeros((n, d), np.float32), np.ones(n, np.float32)
    X, U, W = dev(x), dev(u), dev(w)
    Z = torch.zeros_like(X)
    G = [torch.zeros_like(X) for _ in range(L)]
    eng = sgp.SGP(n, d, peers=peers)
    # first call outside the capture: it sets up the library's device tables (allocations)
    Xs, Us, Ws, Zs = X.clone(), U.clone(), W.clone(), Z.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        eng.step(Xs, Ws, Us, G[0], Zs, 0.05, 0.9, 0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for k in range(L):
            eng.step(X, W, U, G[k], Z, 0.05, 0.9, k)
    for rep in range(4):
        gs = [(0.2 * rng.standard_normal((n, d))).astype(np.float32) for _ in range(L)]
        for k in range(L):
            G[k].copy_(dev(gs[k]))                        # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in range(L):
            zo = O.step(O.mixing_matrix(n, peers, k, np.float32), x, w, u, gs[k], 0.05, 0.9)
        assert np.array_equal(host(X), x), "x after replay %d" % rep
        assert np.array_equal(host(U), u), "u after replay %d" % rep
        assert np.array_equal(host(Z), zo), "z after replay %d" % rep
        assert np.array_equal(host(W), w)
    # and eager calls still work afterwards
    g = (0.2 * rng.standard_normal((n, d))).astype(np.float32)
    eng.step(X, W, U, dev(g), Z, 0.05, 0.9, 0)
    zo = O.step(O.mixing_matrix(n, peers, 0, np.float32), x, w, u, g, 0.05, 0.9)
    assert np.array_equal(host(Z), zo)
    eng.close()
