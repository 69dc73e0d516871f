"""Pins of the storage-experiment oracle (oracle/sgp_oracle.c: sgpo_float_to_bf16, sgpo_step_bf16).
The experiment is not in the paper, so the pins are what the format and the mathematics fix: the
rounding against torch's own bfloat16 conversion and against hand-made ties, and the step by
reduction to the already pinned float32 step on the widened inputs."""
import numpy as np
import torch

from oracle import sgp_oracle as O


def widen(h):
    return (h.astype(np.uint32) << 16).view(np.float32)


def torch_round(f):
    t = torch.from_numpy(np.ascontiguousarray(f, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def oracle_round(f):
    return np.array([O.float_to_bf16(v) for v in np.asarray(f, dtype=np.float32).ravel()], dtype=np.uint16)


def test_every_bfloat16_value_survives_a_round_trip():
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    f = widen(h)
    back = oracle_round(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], h[~nan])
    assert np.all(np.isnan(widen(back[nan])))                  # NaN stays NaN


def test_rounding_matches_torch_on_random_and_special_values():
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 1 << 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    f = bits.view(np.float32)
    f = f[~np.isnan(f)]
    special = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 3.3895314e38, 3.4028235e38, 1e-45, 1.17549435e-38,
                        65504.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7], dtype=np.float32)
    f = np.concatenate([f, special])
    assert np.array_equal(oracle_round(f), torch_round(f))


def test_ties_go_to_the_even_neighbour_and_the_top_overflows_to_infinity():
    one = 0x3f80
    assert O.float_to_bf16(1.0) == one
    assert O.float_to_bf16(1.0 + 2.0 ** -8) == one               # half-way between 1 and 1 + 2^-7: even is 1
    assert O.float_to_bf16(1.0 + 2.0 ** -7 + 2.0 ** -8) == one + 2   # half-way between odd and even: up
    assert O.float_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -20) == one + 1  # just above the tie: up
    assert O.float_to_bf16(1.0 + 2.0 ** -8 - 2.0 ** -20) == one      # just below: down
    assert O.float_to_bf16(-(1.0 + 2.0 ** -8)) == 0x8000 | one
    big = np.float32(3.3895314e38)                               # largest finite bfloat16, 0x7f7f
    assert O.float_to_bf16(big) == 0x7f7f
    assert O.float_to_bf16(np.float32(3.4028235e38)) == 0x7f80   # float max is past the last tie: infinity
    assert np.isnan(O.bf16_to_float(O.float_to_bf16(float("nan"))))


def _case(n, d, seed, peers=1):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    u32 = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    g32 = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    w = (0.5 + rng.random(n)).astype(np.float32)
    return x, u32, torch_round(g32), w


def test_step_reduces_to_the_float32_step_on_the_widened_gradient():
    for n, d, k in ((4, 33, 0), (8, 17, 2), (5, 9, 1), (32, 7, 4)):
        x, u, g16, w = _case(n, d, n + k)
        P = O.mixing_matrix(n, 1, k, np.float32)
        x1, u1, w1 = x.copy(), u.copy(), w.copy()
        z16 = O.step_bf16(P, x1, w1, u1, g16, 0.1, 0.9)
        x2, u2, w2 = x.copy(), u.copy(), w.copy()
        z2 = O.step(P, x2, w2, u2, widen(g16), 0.1, 0.9)
        assert np.array_equal(x1, x2) and np.array_equal(u1, u2) and np.array_equal(w1, w2)
        assert np.array_equal(z16, torch_round(z2))


def test_step_with_sixteen_bit_momentum_rounds_only_what_it_stores():
    for n, d, k in ((4, 33, 0), (16, 21, 3)):
        x, u, g16, w = _case(n, d, 7 * n + k)
        u16 = torch_round(u)
        P = O.mixing_matrix(n, 1, k, np.float32)
        x1, w1, ua = x.copy(), w.copy(), u16.copy()
        z16 = O.step_bf16(P, x1, w1, ua, g16, 0.05, 0.9)
        x2, w2, ub = x.copy(), w.copy(), widen(u16).copy()
        z2 = O.step(P, x2, w2, ub, widen(g16), 0.05, 0.9)
        assert np.array_equal(x1, x2)                      # x uses the momentum as computed, unrounded
        assert np.array_equal(ua, torch_round(ub))         # the stored momentum is its rounding
        assert np.array_equal(z16, torch_round(z2))
        # and a second iteration starts from the rounded momentum
        z16b = O.step_bf16(P, x1, w1, ua, g16, 0.05, 0.9)
        ub = widen(torch_round(ub)).copy()
        z2b = O.step(P, x2, w2, ub, widen(g16), 0.05, 0.9)
        assert np.array_equal(x1, x2) and np.array_equal(z16b, torch_round(z2b))


def test_sixteen_bit_z_is_within_half_a_unit_in_the_eighth_bit_of_the_float32_z():
    x, u, g16, w = _case(8, 1000, 3)
    P = O.mixing_matrix(8, 1, 0, np.float32)
    x2, u2, w2 = x.copy(), u.copy(), w.copy()
    z32 = O.step(P, x2, w2, u2, widen(g16), 0.1, 0.9)
    z16 = O.step_bf16(P, x, w, u, g16, 0.1, 0.9)
    assert np.all(np.abs(widen(z16) - z32) <= 2.0 ** -8 * np.abs(z32))
