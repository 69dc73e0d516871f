"""GPU parity of sgp_step_bf16 (bandwidth experiment: g and z, optionally the momentum, stored as
bfloat16; arithmetic unchanged) against the oracle twin that rounds at the same stores: x, w, the
momentum and the 16-bit patterns of z must be identical."""
import numpy as np
import pytest
import torch

from oracle import sgp_oracle as O
import paper_1811_10792_amd as sgp
from paper_1811_10792_amd import binding, synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda"
GZ, GUZ = binding.SGP_STORE_BF16_GZ, binding.SGP_STORE_BF16_GZ | binding.SGP_STORE_BF16_U


def to_bits(t):
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def round_bits(f):
    return to_bits(torch.from_numpy(np.ascontiguousarray(f, dtype=np.float32)).to(torch.bfloat16))


def run(n, d, ld, storage, iters, seed, w_spread=False, offset=0, k0=0, mom=0.9, gamma=0.1):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    u32 = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    w = (0.5 + rng.random(n)).astype(np.float32) if w_spread else np.ones(n, np.float32)
    u16mode = bool(storage & binding.SGP_STORE_BF16_U)

    def padded(a, dtype_bits):
        """[n, ld] device tensor holding a in its first d columns, starting `offset` elements into a
        larger allocation (offset != 0 breaks the 16-byte alignment)."""
        if dtype_bits:
            full = torch.full((n * ld + offset,), 1.5, dtype=torch.bfloat16, device=DEV)
            view = full[offset:offset + n * ld].view(n, ld)
            view[:, :d] = bf16_dev(a)
        else:
            full = torch.full((n * ld + offset,), 3.5, dtype=torch.float32, device=DEV)
            view = full[offset:offset + n * ld].view(n, ld)
            view[:, :d] = torch.from_numpy(a).to(DEV)
        return full, view
    _, X = padded(x, False)
    uo = round_bits(u32) if u16mode else u32.copy()
    _, U = padded(uo, u16mode)
    _, G = padded(np.zeros((n, d), np.uint16), True)
    _, Z = padded(np.zeros((n, d), np.uint16), True)
    W = torch.from_numpy(w).to(DEV)
    eng = sgp.SGP(n, d, ld)
    xo, wo = x.copy(), w.copy()
    for it in range(iters):
        k = k0 + it
        g16 = round_bits((0.1 * rng.standard_normal((n, d))).astype(np.float32))
        G[:, :d] = bf16_dev(g16)
        eng.step_bf16(X, W, U, G, Z, gamma, mom, k, storage)
        z16 = O.step_bf16(O.mixing_matrix(n, 1, k, np.float32), xo, wo, uo, g16, gamma, mom)
        tag = "n=%d d=%d ld=%d storage=%d k=%d" % (n, d, ld, storage, k)
        assert np.array_equal(X[:, :d].cpu().numpy(), xo), "x " + tag
        assert np.array_equal(W.cpu().numpy(), wo), "w " + tag
        got_u = to_bits(U[:, :d].contiguous()) if u16mode else U[:, :d].cpu().numpy()
        assert np.array_equal(got_u, uo), "u " + tag
        assert np.array_equal(to_bits(Z[:, :d].contiguous()), z16), "z " + tag
    if ld > d:                                                   # padding columns stay untouched
        assert bool((X[:, d:] == 3.5).all()) and bool((Z[:, d:].float() == 1.5).all())
    assert eng.last_step_kernel() == "k_step_one_peer_h16"
    eng.close()


@pytest.mark.parametrize("storage", [GZ, GUZ])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 16, 32, 33])
def test_node_counts(n, storage):
    L = max(1, (n - 1).bit_length())
    run(n, 4104, 4104, storage, L + 1, seed=n + storage, w_spread=(n % 2 == 1))


@pytest.mark.parametrize("storage", [GZ, GUZ])
@pytest.mark.parametrize("d,ld,offset", [(1, 8, 0), (7, 8, 0), (8, 8, 0), (1037, 1040, 0), (1037, 1037, 0),
                                         (2048, 2048, 2), (5000, 5120, 8), (520, 520, 4), (66000, 66048, 0)])
def test_ragged_sizes_padding_and_alignment(d, ld, offset, storage):
    run(8, d, ld, storage, 4, seed=d + offset, w_spread=True, offset=offset, k0=1)


def test_error_paths():
    n, d = 8, 64
    X = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    U = torch.zeros_like(X)
    W = torch.ones(n, dtype=torch.float32, device=DEV)
    G = torch.zeros((n, d), dtype=torch.bfloat16, device=DEV)
    Z = torch.zeros_like(G)
    for kw in (dict(peers=2), dict(delay=1), dict(topology=binding.SGP_TOPO_COMPLETE)):
        eng = sgp.SGP(n, d, **kw)
        with pytest.raises(sgp.SgpError) as e:
            eng.step_bf16(X, W, U, G, Z, 0.1, 0.9, 0, GZ)
        assert e.value.status == binding.SGP_ERR_UNSUPPORTED
        eng.close()
    eng = sgp.SGP(n, d)
    with pytest.raises(sgp.SgpError) as e:
        eng.step_bf16(X, W, U, G, Z, 0.1, 0.0, 0, GZ)              # Alg. 1 is not part of the experiment
    assert e.value.status == binding.SGP_ERR_UNSUPPORTED
    lib = binding.load_library()
    assert lib.sgp_step_bf16(eng._h, X.data_ptr(), W.data_ptr(), U.data_ptr(), G.data_ptr(), Z.data_ptr(),
                             0.1, 0.9, 0, 2, None) == binding.SGP_ERR_INVALID_ARG      # U without G, Z
    assert lib.sgp_step_bf16(eng._h, X.data_ptr(), W.data_ptr(), U.data_ptr(), G.data_ptr() + 1, Z.data_ptr(),
                             0.1, 0.9, 0, 1, None) == binding.SGP_ERR_ALIGNMENT
    torch.cuda.synchronize()
    assert bool((X == 0).all()) and bool((W == 1).all())
    eng.close()


@pytest.mark.parametrize("name", ["h1_n32_resnet50_bf16_gz", "h2_n32_resnet50_bf16_guz"])
def test_full_size_spot_check(name):
    """ResNet-50-sized state in the benchmark's launch configuration; the oracle twin recomputes a
    sample of coordinates including the first tile, the ragged tail and the XCD share boundaries."""
    wl = syn.WORKLOADS[name]
    n, d = wl.n, wl.d
    ld = syn.padded_ld(d)
    storage = GUZ if wl.storage == "bf16_guz" else GZ
    u16mode = storage == GUZ
    X = syn.device_normal(n, ld, wl.x_std, wl.seed, 3)
    U = syn.device_normal(n, ld, wl.grad_std, wl.seed, 6)
    if u16mode:
        U = U.to(torch.bfloat16)
    W = torch.ones(n, dtype=torch.float32, device=DEV)
    Z = torch.empty((n, ld), dtype=torch.bfloat16, device=DEV)
    around = syn.partition_boundaries(d, ld, n, 256)              # 256 coordinates per block
    cols = syn.sample_columns(d, 2000, wl.seed, around=around, halo=128)
    cidx = torch.from_numpy(cols).to(DEV)
    xo = X[:, cidx].cpu().numpy()
    uo = to_bits(U[:, cidx].contiguous()) if u16mode else U[:, cidx].cpu().numpy()
    wo = np.ones(n, np.float32)
    eng = sgp.SGP(n, d, ld)
    for k in range(3):
        G = syn.device_normal(n, ld, wl.grad_std, wl.seed, 100 + k).to(torch.bfloat16)
        eng.step_bf16(X, W, U, G, Z, wl.gamma, wl.momentum, k, storage)
        z16 = O.step_bf16(O.mixing_matrix(n, 1, k, np.float32), xo, wo, uo, to_bits(G[:, cidx].contiguous()),
                          wl.gamma, wl.momentum)
        assert np.array_equal(X[:, cidx].cpu().numpy(), xo), "x k=%d" % k
        got_u = to_bits(U[:, cidx].contiguous()) if u16mode else U[:, cidx].cpu().numpy()
        assert np.array_equal(got_u, uo), "u k=%d" % k
        assert np.array_equal(to_bits(Z[:, cidx].contiguous()), z16), "z k=%d" % k
        del G
    eng.close()
