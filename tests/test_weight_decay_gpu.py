"""GPU parity of weight decay fused into the local step (hyperparameter appendix: weight decay
with Nesterov momentum), on the de-biased parameters or on the numerator, through every step kernel:
bit-exact against the float32 oracle."""
import numpy as np
import pytest
import torch

from oracle import sgp_oracle as O
import paper_1811_10792_amd as sgp
from paper_1811_10792_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def run(n, d, peers, tau, topology, on_x, mom, seed, iters=5, w_spread=True, biased=False, stats=False,
        wd=0.02):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    u = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    w = (0.5 + rng.random(n)).astype(np.float32) if w_spread else np.ones(n, np.float32)
    nest = mom != 0.0
    X, U, W = dev(x), dev(u), dev(w)
    G, Z = torch.zeros_like(X), torch.zeros_like(X)
    eng = sgp.SGP(n, d, topology=topology, peers=peers, delay=tau)
    eng.set_weight_decay(wd, on_numerator=on_x)
    if biased:
        eng.set_biased(True)
    st = O.OsgpState(n, d, np.float32, tau) if tau else None
    oracle_on_x = on_x or biased
    for k in range(iters):
        g = (0.3 * rng.standard_normal((n, d))).astype(np.float32)
        G.copy_(dev(g))
        if stats:
            eng.step_stats(X, W, U if nest else None, G, Z, 0.05, mom, k)
        else:
            eng.step(X, W, U if nest else None, G, Z, 0.05, mom, k)
        if topology == binding.SGP_TOPO_COMPLETE:
            P = np.full((n, n), np.float32(1.0) / np.float32(n), dtype=np.float32)
        else:
            P = O.mixing_matrix(n, peers, k // max(1, tau), np.float32)
        if tau:
            zo = O.step_osgp(P, x, w, u if nest else None, g, 0.05, mom, st, k, nesterov=nest,
                             biased=biased, wd=wd, wd_on_x=oracle_on_x)
        else:
            zo = O.step(P, x, w, u if nest else None, g, 0.05, mom, nesterov=nest, wd=wd,
                        wd_on_x=oracle_on_x)
            if biased:
                zo = x.copy()
        tag = "n=%d peers=%d tau=%d topo=%d on_x=%s k=%d" % (n, peers, tau, topology, on_x, k)
        assert np.array_equal(host(W), w), "w " + tag
        assert np.array_equal(host(X), x), "x " + tag
        assert np.array_equal(host(Z), zo), "z " + tag
        if nest:
            assert np.array_equal(host(U), u), "u " + tag
    eng.close()


@pytest.mark.parametrize("on_x", [False, True])
@pytest.mark.parametrize("peers,tau,topology", [(1, 0, 0), (2, 0, 0), (1, 1, 0), (2, 1, 0), (2, 3, 0),
                                                (1, 0, binding.SGP_TOPO_COMPLETE)])
def test_weight_decay_through_every_step_kernel(peers, tau, topology, on_x):
    run(8, 2052, peers, tau, topology, on_x, 0.9, seed=3 + peers + tau)
    run(5, 1027, peers, tau, topology, on_x, 0.0, seed=4 + peers + tau)       # scalar path, SGD


@pytest.mark.parametrize("n", [16, 32, 12])
def test_weight_decay_in_the_fused_statistics_kernel(n):
    run(n, 4096, 1, 0, 0, False, 0.9, seed=n, stats=True)
    run(n, 4096, 1, 0, 0, True, 0.9, seed=n + 1, stats=True, w_spread=False)


def test_weight_decay_with_the_biased_form_uses_the_numerator():
    run(8, 1024, 1, 1, 0, False, 0.9, seed=70, biased=True, w_spread=False)


def test_weight_decay_can_be_switched_off_again():
    n, d = 4, 256
    rng = np.random.default_rng(5)
    x = rng.standard_normal((n, d)).astype(np.float32)
    g = rng.standard_normal((n, d)).astype(np.float32)
    eng = sgp.SGP(n, d)
    outs = []
    for wd in (0.1, 0.0):
        X, W, G = dev(x), dev(np.ones(n, np.float32)), dev(g)
        Z = torch.zeros_like(X)
        eng.set_weight_decay(wd)
        eng.step(X, W, None, G, Z, 0.1, 0.0, 0)
        xo, wo = x.copy(), np.ones(n, np.float32)
        zo = O.step(O.mixing_matrix(n, 1, 0, np.float32), xo, wo, None, g, 0.1, 0.0, nesterov=False, wd=wd)
        assert np.array_equal(host(Z), zo)
        outs.append(host(Z))
    assert not np.array_equal(outs[0], outs[1])
    with pytest.raises(binding.SgpError):
        eng.set_weight_decay(-1.0)
    eng.close()
