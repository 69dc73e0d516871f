"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it rests on.  Together they are chosen so that a dropped term, a
wrong sign, a wrong hop or a transposed mixing matrix in oracle/sgp_oracle.c fails at least one.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import sgp_oracle as O

F64 = np.float64
F32 = np.float32


# ------------------------------------------------------------------------- fixtures / helpers
def _parse_four_node(golden_dir):
    P = []
    eqs = {}
    with open(os.path.join(golden_dir, "four_node_mixing_matrix.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "P":
                P.append([float(Fraction(v)) for v in t[1:]])
            elif t[0] == "E":
                recv = int(t[1])
                eqs[recv] = [(float(Fraction(s.split("*")[0])), int(s.split("*")[1])) for s in t[3:]]
    return np.array(P, dtype=F64), eqs


def _facts(golden_dir):
    out = {"NEIGHBOUR": [], "COLUMN": [], "TWOPEER": [], "EXACT": [], "CONTRACTION": []}
    with open(os.path.join(golden_dir, "exponential_graph_facts.txt")) as f:
        for line in f:
            t = line.split()
            if t and t[0] in out:
                out[t[0]].append(t[1:])
    return out


def _random_column_stochastic(rng, n, density=0.5):
    """Random sparse column-stochastic matrix with a positive diagonal (every node keeps a share)."""
    M = rng.random((n, n)) * (rng.random((n, n)) < density)
    M[np.arange(n), np.arange(n)] = rng.random(n) + 0.1
    return np.ascontiguousarray(M / M.sum(0, keepdims=True))


def _state(rng, n, d, dtype=F64):
    x = rng.standard_normal((n, d)).astype(dtype)
    u = rng.standard_normal((n, d)).astype(dtype)
    g = rng.standard_normal((n, d)).astype(dtype)
    w = (0.5 + rng.random(n)).astype(dtype)
    return x, w, u, g


# --------------------------------------------------- topology: printed facts (Appendix A)
def test_eight_node_neighbours_printed(golden_dir):
    for n, node, expo, nb in _facts(golden_dir)["NEIGHBOUR"]:
        n, node, expo, nb = int(n), int(node), int(expo), int(nb)
        P = O.mixing_matrix(n, 1, expo)             # iteration k = expo uses hop 2^expo
        col = P[:, node]                            # column = what `node` sends
        assert set(np.nonzero(col)[0]) == {node, nb}
        assert col[nb] == 0.5 and col[node] == 0.5
        if 2 * 2 ** expo != n:                      # directed: the neighbour does not send back
            assert P[node, nb] == 0.0               # (hop n/2 is its own reverse)


def test_column_structure_printed(golden_dir):
    for peers, nnz, val in _facts(golden_dir)["COLUMN"]:
        peers, nnz, val = int(peers), int(nnz), float(Fraction(val))
        for n in (8, 16, 32):
            for k in range(12):
                P = O.mixing_matrix(n, peers, k)
                assert ((P != 0).sum(0) == nnz).all()
                assert np.allclose(P[P != 0], val, rtol=0, atol=1e-16)
                # balanced load: every node also RECEIVES the same number of messages
                assert ((P != 0).sum(1) == nnz).all()


def test_two_peer_window_printed(golden_dir):
    n = 8
    for k, ea, eb in _facts(golden_dir)["TWOPEER"]:
        k, ea, eb = int(k), int(ea), int(eb)
        P = O.mixing_matrix(n, 2, k)
        for i in range(n):
            assert set(np.nonzero(P[:, i])[0]) == {i, (i + 2 ** ea) % n, (i + 2 ** eb) % n}


def test_schedule_cycles_back_to_start():
    # "eventually returning to the beginning of the list before cycling through the peers again"
    for n in (2, 3, 4, 5, 8, 12, 16, 32):
        L = (n - 1).bit_length()
        for peers in (1, 2):
            for k in range(2 * L + 1):
                assert np.array_equal(O.mixing_matrix(n, peers, k), O.mixing_matrix(n, peers, k + L))
        hops = {int(np.nonzero(O.mixing_matrix(n, 1, k)[:, 0])[0].max()) for k in range(L)}
        assert hops == {2 ** r for r in range(L)}   # all of 2^0 .. 2^floor(log2(n-1)) are used


def test_one_peer_matrix_is_half_identity_plus_half_shift():
    # independent construction with numpy's roll: receiver (i+h) mod n hears sender i
    for n in (2, 3, 4, 7, 8, 16, 32, 33):
        L = (n - 1).bit_length()
        for k in range(2 * L):
            h = 2 ** (k % L)
            shift = np.roll(np.eye(n), h, axis=0)    # shift[(i+h)%n, i] = 1
            assert np.array_equal(O.mixing_matrix(n, 1, k), 0.5 * np.eye(n) + 0.5 * shift)


@pytest.mark.parametrize("dtype", [F64, F32])
def test_columns_sum_to_one(dtype):
    # "column stochastic (all columns sum to 1)"
    for n in range(1, 34):
        for peers in (1, 2, 3):
            for k in range(0, 7):
                P = O.mixing_matrix(n, peers, k, dtype)
                tol = 0 if dtype == F64 and peers == 1 else 4e-8 if dtype == F32 else 2e-16
                assert np.abs(P.astype(F64).sum(0) - 1.0).max() <= tol
    assert O.mixing_matrix(1, 1, 0).tolist() == [[1.0]]
    assert O.mixing_matrix(1, 2, 5).tolist() == [[1.0]]
    # out-neighbourhood is a set: with n = 2 both "peers" are the same node
    assert np.array_equal(O.mixing_matrix(2, 2, 0), O.mixing_matrix(2, 1, 0))


# ------------------------------------------ exact averaging ("Decentralized averaging errors")
def test_exact_average_after_one_cycle_printed(golden_dir):
    for n, its in _facts(golden_dir)["EXACT"]:
        n, its = int(n), int(its)
        for k0 in range(0, 7):
            prod = np.eye(n)
            for k in range(k0, k0 + its):
                prod = O.mixing_matrix(n, 1, k) @ prod
            assert np.array_equal(prod, np.full((n, n), 1.0 / n))       # exactly 2^-5 everywhere
            s = np.linalg.svd(prod, compute_uv=False)
            assert s[1] < 1e-15                                         # lambda_2 = 0
            short = np.eye(n)
            for k in range(k0, k0 + its - 1):
                short = O.mixing_matrix(n, 1, k) @ short
            assert (short == 0).any()                                   # one step fewer is not enough


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_step_reaches_exact_average_with_gamma_zero(n):
    rng = np.random.default_rng(n)
    d = 5
    L = (n - 1).bit_length()
    x0 = rng.standard_normal((n, d))
    w0 = 0.5 + rng.random(n)
    for k0 in (0, 3):
        x, w = x0.copy(), w0.copy()
        u, g = np.zeros((n, d)), rng.standard_normal((n, d))
        for k in range(k0, k0 + L):
            z = O.step(O.mixing_matrix(n, 1, k), x, w, u, g, 0.0, 0.0, nesterov=False)
        target = x0.sum(0) / w0.sum()        # general w^(0) > 0: ratio of sums
        assert np.abs(z - target).max() < 1e-14
        assert np.abs(w - w0.mean()).max() < 1e-15


# --------------------------------------------- worked 4-node example (printed matrix + equations)
def test_four_node_example_printed(golden_dir):
    P, eqs = _parse_four_node(golden_dir)
    assert np.abs(P.sum(0) - 1).max() < 1e-15          # "the matrix is column stochastic"
    rng = np.random.default_rng(7)
    d = 6
    x0 = rng.standard_normal((4, d))
    for dtype, tol in ((F64, 1e-15), (F32, 3e-7)):
        x = x0.astype(dtype)
        w = np.ones(4, dtype)
        g = np.zeros((4, d), dtype)
        z = O.step(np.ascontiguousarray(P.astype(dtype)), x, w, None, g, 0.0, 0.0, nesterov=False)
        for recv, terms in eqs.items():                # the paper's four printed equations
            want = sum(coef * x0[snd] for coef, snd in terms)
            assert np.abs(x[recv] - want).max() <= tol * 4
        # "similar equations can be written for the push-sum weights": w = P 1
        want_w = np.array([Fraction(1, 2) + Fraction(1, 3), Fraction(1, 2) * 2 + Fraction(1, 3),
                           Fraction(1), Fraction(1, 2) + Fraction(1, 3)], dtype=object)
        assert np.abs(w.astype(F64) - want_w.astype(F64)).max() <= tol
        assert np.abs(z.astype(F64) - x.astype(F64) / w.astype(F64)[:, None]).max() <= tol * 4


# ------------------------------------------------------- column-stochastic conservation
@pytest.mark.parametrize("nesterov", [False, True])
def test_mass_conservation(nesterov):
    # 1^T P = 1^T  =>  sum_i x_i^(k+1) = sum_i (x_i - gamma * update_i),  sum_i w_i constant
    rng = np.random.default_rng(11)
    for n in (1, 2, 3, 5, 8, 13):
        d = 9
        P = _random_column_stochastic(rng, n)
        x, w, u, g = _state(rng, n, d)
        gamma, m = 0.3, 0.8
        x0, w0, u0 = x.copy(), w.copy(), u.copy()
        O.step(P, x, w, u, g, gamma, m, nesterov=nesterov)
        if nesterov:
            u_new = m * u0 + g
            upd = m * u_new + g
            assert np.abs(u - u_new).max() < 1e-15
        else:
            upd = g
            assert np.array_equal(u, u0)               # Alg. 1 has no momentum buffer
        assert np.abs(x.sum(0) - (x0 - gamma * upd).sum(0)).max() < 1e-13
        assert abs(w.sum() - w0.sum()) < 1e-14


def test_consensus_is_a_fixed_point_of_the_mix():
    # if every numerator is w_j * c, a gamma = 0 step returns z_i = c for any column-stochastic P
    rng = np.random.default_rng(12)
    for n in (2, 4, 7):
        d = 8
        P = _random_column_stochastic(rng, n)
        c = rng.standard_normal(d)
        w = 0.5 + rng.random(n)
        x = w[:, None] * c[None, :]
        z = O.step(P, x, w, np.zeros((n, d)), rng.standard_normal((n, d)), 0.0, 0.9, nesterov=False)
        assert np.abs(z - c[None, :]).max() < 1e-14


def test_brute_force_dense_product():
    # the step is X <- (X - gamma * update) P^T written with numpy's matmul
    rng = np.random.default_rng(13)
    for n in (1, 2, 3, 4, 5, 8):
        L = max(1, (n - 1).bit_length())
        for peers in (1, 2):
            for k in range(2 * L):
                d = 7
                P = O.mixing_matrix(n, peers, k)
                x, w, u, g = _state(rng, n, d)
                gamma, m = 0.05, 0.9
                un = m * u + g
                xh = x - gamma * (m * un + g)
                want_x, want_w = P @ xh, P @ w
                z = O.step(P, x, w, u, g, gamma, m, nesterov=True)
                assert np.abs(x - want_x).max() < 1e-14
                assert np.abs(w - want_w).max() < 1e-15
                assert np.abs(z - want_x / want_w[:, None]).max() < 1e-13


def _one_peer_matrix(n, dest):
    """Column-stochastic one-peer matrix: node i keeps half and sends half to dest[i]."""
    P = np.zeros((n, n))
    for i in range(n):
        P[i, i] += 0.5
        P[dest[i], i] += 0.5
    return P


def test_printed_contraction_factors_of_other_one_peer_schemes(golden_dir):
    # "Decentralized averaging errors": sigma_2^2 of the product of five mixing matrices is the number
    # the paper prints for each scheme (to its one printed digit); the oracle's mix applies exactly
    # that product and, for the doubly stochastic scheme, contracts the worst-case start by it
    rng = np.random.default_rng(2024)
    for scheme, n, its, printed in _facts(golden_dir)["CONTRACTION"]:
        n, its, printed = int(n), int(its), float(printed)
        trials = 1 if scheme == "complete_cycle" else 200
        factors = []
        for _ in range(trials):
            Ps = []
            for k in range(its):
                if scheme == "complete_cycle":
                    dest = [(i + k + 1) % n for i in range(n)]
                elif scheme == "random_exponential":
                    dest = [(i + 2 ** int(rng.integers(5))) % n for i in range(n)]
                else:
                    dest = [(i + 1 + int(rng.integers(n - 1))) % n for i in range(n)]
                Ps.append(_one_peer_matrix(n, dest))
            prod = np.eye(n)
            for P in Ps:
                prod = P @ prod
            _, sv, vt = np.linalg.svd(prod)
            y0 = np.ascontiguousarray(vt[1][:, None] * np.ones((1, 3)))   # worst-case start, 3 coordinates
            y, w = y0.copy(), np.ones(n)
            for P in Ps:
                O.step(np.ascontiguousarray(P), y, w, None, np.zeros_like(y), 0.0, 0.0, nesterov=False)
            assert np.abs(y - prod @ y0).max() < 1e-14            # the oracle applies exactly this product
            if scheme == "complete_cycle":
                # doubly stochastic: the average is kept and the worst-case start contracts by sigma_2^2
                e0 = ((y0 - y0.mean(0)) ** 2).sum()
                assert abs(((y - y.mean(0)) ** 2).sum() / e0 - sv[1] ** 2) < 1e-12
                assert np.abs(y.mean(0) - y0.mean(0)).max() < 1e-15 and np.abs(w - 1).max() < 1e-15
            factors.append(sv[1] ** 2)
        assert abs(np.mean(factors) - printed) < 0.05, (scheme, np.mean(factors))


def test_deviation_plateau_is_proportional_to_the_step_size():
    # "Parameter deviations" / the consensus lemma behind it: nodes converge to a neighbourhood of
    # the average whose size is proportional to the step size.  Heterogeneous quadratics with
    # gradient noise: halving gamma halves the stationary mean distance to the node-wise average.
    def plateau(gamma, n=8, d=64, iters=600):
        rng = np.random.default_rng(5)
        h = 0.5 + 1.5 * rng.random((n, d))
        c = rng.standard_normal((n, d))
        x = rng.standard_normal((n, d))
        w, z, acc = np.ones(n), x.copy(), []
        for k in range(iters):
            g = h * (z - c) + 0.1 * rng.standard_normal((n, d))
            z = O.step(O.mixing_matrix(n, 1, k), x, w, None, g, gamma, 0.0, nesterov=False)
            if k >= iters - 200:
                acc.append(O.consensus_stats(z, w)[1]["mean"])
        return float(np.mean(acc))
    p1, p2, p4 = plateau(0.1), plateau(0.05), plateau(0.025)
    assert 1.8 < p1 / p2 < 2.2 and 1.8 < p2 / p4 < 2.2


# ------------------------------------------------- reductions to textbook / library routines
@pytest.mark.parametrize("nesterov,m", [(False, 0.0), (True, 0.9), (True, 0.5)])
def test_all_to_all_equals_parallel_sgd_library(nesterov, m):
    # every entry of P equal to 1/n and identical initial values: SGP is parallel SGD with an
    # exact gradient average.  The comparison optimiser is torch.optim.SGD on the CPU.
    n, d, gamma, iters = 6, 10, 0.07, 12
    rng = np.random.default_rng(14)
    h = 0.5 + 1.5 * rng.random((n, d))
    c = rng.standard_normal((n, d))
    x_init = rng.standard_normal(d)
    P = np.full((n, n), 1.0 / n)
    x = np.tile(x_init, (n, 1))
    w = np.ones(n)
    u = np.zeros((n, d))
    z = x.copy()
    p = torch.tensor(x_init.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=m if nesterov else 0.0, nesterov=nesterov)
    for _ in range(iters):
        g = h * (z - c)                                    # each node's gradient at its z_i
        z = O.step(P, x, w, u, g, gamma, m, nesterov=nesterov)
        opt.zero_grad()
        p.grad = torch.tensor((h * (p.detach().numpy()[None, :] - c)).mean(0))
        opt.step()
        assert np.abs(z - p.detach().numpy()[None, :]).max() < 1e-12
    assert np.abs(w - 1).max() < 1e-15


def test_single_node_is_plain_nesterov_sgd_library():
    d, gamma, m = 16, 0.1, 0.9
    rng = np.random.default_rng(15)
    x = rng.standard_normal((1, d))
    p = torch.tensor(x[0].copy(), requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=m, nesterov=True)
    w, u = np.ones(1), np.zeros((1, d))
    P = O.mixing_matrix(1, 1, 0)
    for k in range(8):
        g = rng.standard_normal((1, d))
        z = O.step(P, x, w, u, g, gamma, m, nesterov=True)
        p.grad = torch.tensor(g[0].copy())
        opt.step()
        assert np.abs(z[0] - p.detach().numpy()).max() < 1e-13
        assert np.abs(u[0] - opt.state[p]["momentum_buffer"].numpy()).max() < 1e-13


@pytest.mark.parametrize("nesterov,m", [(False, 0.0), (True, 0.9)])
def test_weight_decay_is_the_library_optimizers(nesterov, m):
    # one node: x = z, and SGP with weight decay is torch.optim.SGD(weight_decay=...)
    d, gamma, wd = 12, 0.1, 0.05
    rng = np.random.default_rng(41)
    x = rng.standard_normal((1, d))
    p = torch.tensor(x[0].copy(), requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=m, nesterov=nesterov, weight_decay=wd)
    w, u = np.ones(1), np.zeros((1, d))
    for k in range(8):
        g = rng.standard_normal((1, d))
        z = O.step(np.ones((1, 1)), x, w, u, g, gamma, m, nesterov=nesterov, wd=wd, wd_on_x=bool(k & 1))
        p.grad = torch.tensor(g[0].copy())
        opt.step()
        assert np.abs(z[0] - p.detach().numpy()).max() < 1e-13


def test_weight_decay_acts_on_z_or_on_x():
    # equivalent to handing over g + wd * theta, with theta = x / w (default) or x
    rng = np.random.default_rng(42)
    n, d, wd = 5, 7, 0.03
    P = _random_column_stochastic(rng, n)
    x, w, u, g = _state(rng, n, d)
    for on_x in (False, True):
        theta = x if on_x else x / w[:, None]
        xa, wa, ua = x.copy(), w.copy(), u.copy()
        za = O.step(P, xa, wa, ua, g, 0.1, 0.9, wd=wd, wd_on_x=on_x)
        xb, wb, ub = x.copy(), w.copy(), u.copy()
        zb = O.step(P, xb, wb, ub, g + wd * theta, 0.1, 0.9)
        assert np.abs(xa - xb).max() < 1e-15 and np.abs(za - zb).max() < 1e-14
        assert np.abs(ua - ub).max() < 1e-15 and np.array_equal(wa, wb)
        # same through the overlap oracle
        st1, st2 = O.OsgpState(n, d, F64, 2), O.OsgpState(n, d, F64, 2)
        xa, wa, ua = x.copy(), w.copy(), u.copy()
        xb, wb, ub = x.copy(), w.copy(), u.copy()
        for k in range(3):
            th = xb if on_x else xb / wb[:, None]
            gb = g + wd * th
            za = O.step_osgp(P, xa, wa, ua, g, 0.1, 0.9, st1, k, wd=wd, wd_on_x=on_x)
            zb = O.step_osgp(P, xb, wb, ub, gb, 0.1, 0.9, st2, k)
            assert np.abs(xa - xb).max() < 1e-14 and np.abs(za - zb).max() < 1e-13
    # and the two variants differ when w != 1
    xa, wa, ua = x.copy(), w.copy(), u.copy()
    xb, wb, ub = x.copy(), w.copy(), u.copy()
    O.step(P, xa, wa, ua, g, 0.1, 0.9, wd=wd, wd_on_x=False)
    O.step(P, xb, wb, ub, g, 0.1, 0.9, wd=wd, wd_on_x=True)
    assert np.abs(xa - xb).max() > 1e-4


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_local_step_is_the_library_optimizer(wd):
    # every node runs torch.optim.Adam on its numerator with the gradient it was handed; the mix
    # is then the dense product with P (per coordinate)
    rng = np.random.default_rng(43)
    n, d, gamma, b1, b2, eps = 4, 6, 0.01, 0.9, 0.98, 1e-8
    P = _random_column_stochastic(rng, n)
    x = rng.standard_normal((n, d))
    w = np.ones(n)
    m1, m2 = np.zeros((n, d)), np.zeros((n, d))
    params = [torch.tensor(x[i].copy(), requires_grad=True) for i in range(n)]
    opts = [torch.optim.Adam([p], lr=gamma, betas=(b1, b2), eps=eps, weight_decay=wd) for p in params]
    for t in range(1, 7):
        g = rng.standard_normal((n, d))
        for i in range(n):
            with torch.no_grad():
                params[i].copy_(torch.tensor(x[i]))       # the optimiser steps on the numerator
            params[i].grad = torch.tensor(g[i].copy())
            opts[i].step()
        xh = np.stack([p.detach().numpy() for p in params])
        w_ref = P @ w
        z = O.step(P, x, w, m1, g, gamma, 0.0, nesterov=False, wd=wd, wd_on_x=True,
                   adam=O.adam_params(b1, b2, eps, t, F64), v=m2)
        assert np.abs(x - P @ xh).max() < 1e-12
        assert np.abs(w - w_ref).max() < 1e-15
        assert np.abs(z - (P @ xh) / w_ref[:, None]).max() < 1e-12
        for i in range(n):
            st = opts[i].state[params[i]]
            assert np.abs(m1[i] - st["exp_avg"].numpy()).max() < 1e-14
            assert np.abs(m2[i] - st["exp_avg_sq"].numpy()).max() < 1e-14


def test_adam_under_overlap_equals_adam_then_delayed_mix():
    # the overlap oracle with Adam = the same local step followed by the delayed mix: compare with
    # the blocking oracle's local step (P = I gives xh) fed through the tau = 2 message schedule
    rng = np.random.default_rng(44)
    n, d, tau = 5, 3, 2
    x = rng.standard_normal((n, d))
    w = np.ones(n)
    xa, wa, ua, va = x.copy(), w.copy(), np.zeros((n, d)), np.zeros((n, d))
    xb, wb, ub, vb = x.copy(), w.copy(), np.zeros((n, d)), np.zeros((n, d))
    sa, sb = O.OsgpState(n, d, F64, tau), O.OsgpState(n, d, F64, tau)
    for k in range(7):
        g = rng.standard_normal((n, d))
        ad = O.adam_params(0.9, 0.999, 1e-8, k + 1, F64)
        P = O.mixing_matrix(n, 2, k // tau)
        za = O.step_osgp(P, xa, wa, ua, g, 0.05, 0.0, sa, k, nesterov=False, adam=ad, v=va)
        # reference: local Adam step alone (identity mixing), then plain SGD-free overlap step with
        # gamma = 0 on the result
        wtmp = np.ones(n)
        xh = xb.copy()
        O.step(np.eye(n), xh, wtmp, ub, g, 0.05, 0.0, nesterov=False, adam=ad, v=vb)
        xb[:] = xh
        zb = O.step_osgp(P, xb, wb, None, np.zeros((n, d)), 0.0, 0.0, sb, k, nesterov=False)
        assert np.abs(xa - xb).max() < 1e-14 and np.abs(wa - wb).max() < 1e-15
        assert np.abs(za - zb).max() < 1e-13
        assert np.array_equal(ua, ub) and np.array_equal(va, vb)


def test_zero_momentum_reduces_alg3_to_alg1():
    rng = np.random.default_rng(16)
    for dtype in (F64, F32):
        n, d = 8, 33
        P = O.mixing_matrix(n, 1, 2, dtype)
        x, w, u, g = _state(rng, n, d, dtype)
        xa, wa = x.copy(), w.copy()
        za = O.step(P, xa, wa, None, g, 0.1, 0.0, nesterov=False)
        xb, wb, ub = x.copy(), w.copy(), u.copy()
        zb = O.step(P, xb, wb, ub, g, 0.1, 0.0, nesterov=True)
        assert np.array_equal(xa, xb) and np.array_equal(za, zb) and np.array_equal(wa, wb)
        assert np.array_equal(ub, g)                        # u <- 0*u + g


def test_doubly_stochastic_keeps_unit_weights():
    # symmetric/doubly stochastic mixing needs no de-biasing: w stays 1 (also in float32,
    # where 3 * fl(1/3) rounds back to 1)
    for dtype in (F64, F32):
        for n in (4, 8, 16, 32):
            for peers in (1, 2):
                w = np.ones(n, dtype)
                x = np.ones((n, 3), dtype)
                for k in range(7):
                    P = O.mixing_matrix(n, peers, k, dtype)
                    assert np.abs(P.astype(F64).sum(1) - 1).max() < 1e-7
                    z = O.step(P, x, w, None, np.zeros((n, 3), dtype), 0.0, 0.0, nesterov=False)
                    assert (w == 1).all()
                    assert np.array_equal(z, x)


# ---------------------------------------------------------- 1-overlap SGP (Alg. 2, tau = 1)
def _augmented(Pk, n):
    """Augmented 2n x 2n matrix of the delay model with tau = 1: self-messages arrive at once
    (block P_0 = diagonal part), all others one iteration late (block P_1 = off-diagonal part),
    virtual nodes forward everything (identity block)."""
    D = np.diag(np.diag(Pk))
    Off = Pk - D
    return np.block([[D, np.eye(n)], [Off, np.zeros((n, n))]])


@pytest.mark.parametrize("peers", [1, 2])
def test_delay_matches_virtual_node_model(peers):
    rng = np.random.default_rng(17)
    n, d, gamma, m = 8, 5, 0.05, 0.9
    x, w, u, _ = _state(rng, n, d)
    w[:] = 1.0
    u[:] = 0.0
    st = O.Delay1State(n, d, F64)
    X = np.vstack([x.copy(), np.zeros((n, d))])           # virtual nodes start at x = 0, w = 0
    W = np.concatenate([w.copy(), np.zeros(n)])
    U = u.copy()
    total_x0 = X.sum(0).copy()
    drift = np.zeros(d)
    for k in range(9):
        g = rng.standard_normal((n, d))
        P = O.mixing_matrix(n, peers, k)
        A = _augmented(P, n)
        assert np.abs(A.sum(0) - 1).max() < 1e-15         # augmented matrices stay column stochastic
        U = m * U + g
        upd = m * U + g
        XH = X.copy()
        XH[:n] -= gamma * upd                             # virtual nodes take no gradient step
        X, W = A @ XH, A @ W
        drift += gamma * upd.sum(0)
        z = O.step_delay1(P, x, w, u, g, gamma, m, st, nesterov=True)
        assert np.abs(x - X[:n]).max() < 1e-13
        assert np.abs(w - W[:n]).max() < 1e-15
        assert np.abs(z - X[:n] / W[:n, None]).max() < 1e-12
        # conservation counts what is in transit
        assert np.abs(X.sum(0) - (total_x0 - drift)).max() < 1e-12
        assert abs(W.sum() - n) < 1e-14


def test_delay_weight_closed_forms():
    # all nodes share w^(k); one peer:  w^(k+1) = w^(k)/2 + w^(k-1)/2,  w^(1) = 1/2
    #                       two peers: w^(k+1) = w^(k)/3 + 2 w^(k-1)/3, w^(1) = 1/3
    n, d = 16, 2
    for peers, a, b, r in ((1, Fraction(2, 3), Fraction(1, 3), Fraction(-1, 2)),
                           (2, Fraction(3, 5), Fraction(2, 5), Fraction(-2, 3))):
        x, w, u = np.ones((n, d)), np.ones(n), np.zeros((n, d))
        st = O.Delay1State(n, d, F64)
        for k in range(10):
            assert np.abs(w - float(a + b * r ** k)).max() < 1e-15
            z = O.step_delay1(O.mixing_matrix(n, peers, k), x, w, u, np.zeros((n, d)), 0.0, 0.0,
                              st, nesterov=False)
            assert np.abs(z - 1.0).max() < 1e-14           # consensus survives delay only via x / w
            assert np.abs(x - w[:, None]).max() < 1e-15    # while x itself drifts away from 1


def test_first_delayed_step_receives_nothing():
    rng = np.random.default_rng(18)
    n, d = 4, 3
    x, w, u, g = _state(rng, n, d)
    x0, w0 = x.copy(), w.copy()
    st = O.Delay1State(n, d, F64)
    O.step_delay1(O.mixing_matrix(n, 1, 0), x, w, None, g, 0.5, 0.0, st, nesterov=False)
    assert np.abs(x - 0.5 * (x0 - 0.5 * g)).max() < 1e-15
    assert np.abs(w - 0.5 * w0).max() < 1e-16


# ------------------------------------------------ tau-overlap SGP (Alg. 2, tau >= 1), biased form
def _augmented_tau(Pk, n, tau, sending):
    """Augmented n(tau+1) x n(tau+1) matrix of the appendix on message delays, block form: first
    block column = (P_0; P_1; ..; P_tau), identity blocks above the diagonal (virtual nodes forward
    what they hold).  Deterministic reading: self-messages have delay 0, all others delay tau, and
    at an iteration without communication every node keeps everything (P_0 = I)."""
    N = n * (tau + 1)
    A = np.zeros((N, N))
    for r in range(tau):
        A[r * n:(r + 1) * n, (r + 1) * n:(r + 2) * n] = np.eye(n)
    if sending:
        D = np.diag(np.diag(Pk))
        A[:n, :n] = D
        A[tau * n:, :n] = Pk - D
    else:
        A[:n, :n] = np.eye(n)
    return A


@pytest.mark.parametrize("tau", [1, 2, 3])
@pytest.mark.parametrize("peers", [1, 2])
@pytest.mark.parametrize("n", [2, 3, 5, 8])
def test_osgp_matches_virtual_node_model(tau, peers, n):
    rng = np.random.default_rng(100 * tau + 10 * peers + n)
    d, gamma, m = 4, 0.05, 0.9
    x, w, u, _ = _state(rng, n, d)
    u[:] = 0.0
    st = O.OsgpState(n, d, F64, tau)
    X = np.vstack([x.copy()] + [np.zeros((n, d))] * tau)  # virtual nodes start at x = 0, w = 0
    W = np.concatenate([w.copy(), np.zeros(n * tau)])
    U = u.copy()
    total_x0, total_w0 = X.sum(0).copy(), W.sum()
    drift = np.zeros(d)
    for k in range(4 * tau + 3):
        g = rng.standard_normal((n, d))
        sending = k % tau == 0
        P = O.mixing_matrix(n, peers, k // tau)
        A = _augmented_tau(P, n, tau, sending)
        assert np.abs(A.sum(0) - 1).max() < 1e-15         # column stochastic at every iteration
        U = m * U + g
        upd = m * U + g
        XH = X.copy()
        XH[:n] -= gamma * upd
        X, W = A @ XH, A @ W
        drift += gamma * upd.sum(0)
        z = O.step_osgp(P, x, w, u, g, gamma, m, st, k, nesterov=True)
        assert np.abs(x - X[:n]).max() < 1e-13
        assert np.abs(w - W[:n]).max() < 1e-15
        assert np.abs(z - X[:n] / W[:n, None]).max() < 1e-12
        assert np.abs(X.sum(0) - (total_x0 - drift)).max() < 1e-12
        assert abs(W.sum() - total_w0) < 1e-14


def test_osgp_with_tau_one_is_the_one_overlap_oracle():
    rng = np.random.default_rng(31)
    n, d = 8, 33
    for dtype in (F64, F32):
        x, w, u, _ = _state(rng, n, d, dtype)
        xa, wa, ua = x.copy(), w.copy(), u.copy()
        sa, sb = O.Delay1State(n, d, dtype), O.OsgpState(n, d, dtype, 1)
        for k in range(7):
            g = rng.standard_normal((n, d)).astype(dtype)
            P = O.mixing_matrix(n, 2, k, dtype)
            za = O.step_delay1(P, xa, wa, ua, g, 0.1, 0.9, sa)
            zb = O.step_osgp(P, x, w, u, g, 0.1, 0.9, sb, k)
            assert np.array_equal(za, zb) and np.array_equal(xa, x) and np.array_equal(wa, w)
            assert np.array_equal(ua, u)


def test_osgp_weight_closed_form_per_round():
    # tau = 3, one peer: the common weight changes only at sending iterations and, counted in
    # rounds c = ceil(k / tau), follows the tau = 1 recursion: 2/3 + (1/3) (-1/2)^c
    n, d, tau = 8, 2, 3
    x, w = np.ones((n, d)), np.ones(n)
    st = O.OsgpState(n, d, F64, tau)
    for k in range(16):
        c = -(-k // tau)
        assert np.abs(w - float(Fraction(2, 3) + Fraction(1, 3) * Fraction(-1, 2) ** c)).max() < 1e-15
        z = O.step_osgp(O.mixing_matrix(n, 1, k // tau), x, w, None, np.zeros((n, d)), 0.0, 0.0, st, k,
                        nesterov=False)
        assert np.abs(z - 1.0).max() < 1e-14               # de-biased consensus is kept ...
    # ... while the biased form (z = x) reports the drifted numerators
    x, w = np.ones((n, d)), np.ones(n)
    st = O.OsgpState(n, d, F64, tau)
    for k in range(7):
        z = O.step_osgp(O.mixing_matrix(n, 1, k // tau), x, w, None, np.zeros((n, d)), 0.0, 0.0, st, k,
                        nesterov=False, biased=True)
        assert np.array_equal(z, x)
    assert np.abs(z - w[:, None]).max() < 1e-15 and abs(w[0] - 1.0) > 0.2


def test_osgp_between_sends_is_a_local_step():
    rng = np.random.default_rng(32)
    n, d, tau = 4, 3, 4
    x, w, u, g = _state(rng, n, d)
    st = O.OsgpState(n, d, F64, tau)
    O.step_osgp(O.mixing_matrix(n, 1, 0), x, w, None, g, 0.5, 0.0, st, 0, nesterov=False)
    x1, w1 = x.copy(), w.copy()
    g2 = rng.standard_normal((n, d))
    z = O.step_osgp(np.full((n, n), np.nan), x, w, None, g2, 0.5, 0.0, st, 1, nesterov=False)
    assert np.abs(x - (x1 - 0.5 * g2)).max() < 1e-15       # P is not even read
    assert np.array_equal(w, w1)
    assert np.abs(z - x / w[:, None]).max() < 1e-15
    assert st.arrival[0] == tau                            # the first messages are still in flight


# ------------------------------------------------------------------ float32 twin, de-bias
def test_float32_twin_tracks_float64():
    rng = np.random.default_rng(19)
    n, d = 16, 257
    x, w, u, g = _state(rng, n, d, F32)
    for peers in (1, 2):
        xs, ws, us = x.copy(), w.copy(), u.copy()
        xd, wd, ud = x.astype(F64), w.astype(F64), u.astype(F64)
        zs = O.step(O.mixing_matrix(n, peers, 1, F32), xs, ws, us, g, 0.1, 0.9)
        zd = O.step(O.mixing_matrix(n, peers, 1, F64), xd, wd, ud, g.astype(F64), 0.1, 0.9)
        scale = np.abs(x).max() + 0.1 * 2 * np.abs(g).max() + 0.1 * np.abs(u).max()
        assert np.abs(xs - xd).max() <= 8 * 2.0 ** -24 * scale
        assert np.abs(us - ud).max() <= 4 * 2.0 ** -24 * (np.abs(u).max() + np.abs(g).max())
        assert np.abs(zs - zd).max() <= 16 * 2.0 ** -24 * scale / w.min()


def test_debias_is_elementwise_division():
    rng = np.random.default_rng(20)
    x = rng.standard_normal((5, 11)).astype(F32)
    w = (0.5 + rng.random(5)).astype(F32)
    assert np.array_equal(O.debias(x, w), x / w[:, None])   # numpy's float32 division is IEEE too


# ------------------------------------------------------------------ consensus statistics
def test_stats_closed_forms():
    # two nodes placed symmetrically about c: both are exactly ||t|| away from the average
    c = np.array([1.0, -2.0, 3.0, 0.5])
    t = np.array([3.0, 0.0, -4.0, 0.0])
    dist, s = O.consensus_stats(np.stack([c + t, c - t]), np.array([0.25, 1.75]))
    assert np.allclose(dist, [5.0, 5.0], rtol=0, atol=1e-15)
    assert s["max"] == s["min"] == s["mean"] == 5.0 and s["w_sum"] == 2.0
    assert abs(s["zbar_norm"] - np.sqrt((c * c).sum())) < 1e-15
    # one node displaced by v among n identical ones: it is (n-1)/n |v| away, the others |v|/n
    n, d = 5, 7
    rng = np.random.default_rng(21)
    base, v = rng.standard_normal(d), rng.standard_normal(d)
    z = np.tile(base, (n, 1))
    z[2] += v
    dist, s = O.consensus_stats(z, np.ones(n))
    nv = np.linalg.norm(v)
    want = np.full(n, nv / n)
    want[2] = nv * (n - 1) / n
    assert np.allclose(dist, want, rtol=1e-14)
    assert abs(s["max"] - want[2]) < 1e-14 and abs(s["min"] - nv / n) < 1e-14
    assert abs(s["mean"] - want.mean()) < 1e-14


def test_stats_against_numpy():
    rng = np.random.default_rng(22)
    z = rng.standard_normal((9, 1000)).astype(F32)
    w = rng.random(9).astype(F32)
    dist, s = O.consensus_stats(z, w)
    z64 = z.astype(F64)
    want = np.linalg.norm(z64 - z64.mean(0, keepdims=True), axis=1)
    assert np.allclose(dist, want, rtol=1e-13)
    assert abs(s["w_sum"] - w.astype(F64).sum()) < 1e-14
    assert abs(s["zbar_norm"] - np.linalg.norm(z64.mean(0))) < 1e-13


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(23)
    n, d = 8, 4099
    x, w, u, g = _state(rng, n, d, F32)
    P = O.mixing_matrix(n, 2, 3, F32)
    outs = []
    for t in (1, 3):
        O.set_threads(t)
        xs, ws, us = x.copy(), w.copy(), u.copy()
        z = O.step(P, xs, ws, us, g, 0.1, 0.9)
        outs.append((xs, ws, us, z))
    O.set_threads(O.max_threads())
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
