"""GPU checks of the measurement utilities of the C ABI: the plain copy and the structure-free
stream pattern (every written element is the float sum of the elements read at its offset)."""
import numpy as np
import pytest
import torch

import paper_1811_10792_amd as sgp

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_copy_moves_every_byte():
    rng = np.random.default_rng(0)
    src = torch.from_numpy(rng.standard_normal(4 * 100_003).astype(np.float32)).to(DEV)
    dst = torch.zeros_like(src)
    sgp.sgp_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


@pytest.mark.parametrize("nr,nw", [(3, 3), (1, 1), (0, 2), (4, 4), (2, 0), (4, 1)])
def test_stream_pattern_writes_the_sum_of_what_it_reads(nr, nw):
    rng = np.random.default_rng(10 * nr + nw)
    count = 4 * (256 * 37 + 5)                                   # several blocks and a ragged last one
    reads_h = [rng.standard_normal(count).astype(np.float32) for _ in range(nr)]
    reads = [torch.from_numpy(a).to(DEV) for a in reads_h]
    writes = [torch.full((count,), 7.0, dtype=torch.float32, device=DEV) for _ in range(nw)]
    guard = torch.full((count,), 3.0, dtype=torch.float32, device=DEV)
    sgp.sgp_stream_pattern(reads, writes)
    torch.cuda.synchronize()
    want = np.zeros(count, np.float32)
    for a in reads_h:                                            # same order of additions, float32
        want = (want + a).astype(np.float32)
    for w in writes:
        assert np.array_equal(w.cpu().numpy(), want)
    for r, a in zip(reads, reads_h):
        assert np.array_equal(r.cpu().numpy(), a)
    assert (guard == 3.0).all()


def test_stream_pattern_in_place():
    rng = np.random.default_rng(5)
    count = 4 * 1000
    x_h, u_h, g_h = (rng.standard_normal(count).astype(np.float32) for _ in range(3))
    x, u, g = (torch.from_numpy(a).to(DEV) for a in (x_h, u_h, g_h))
    z = torch.zeros_like(x)
    sgp.sgp_stream_pattern([x, u, g], [x, u, z])
    torch.cuda.synchronize()
    want = ((x_h + u_h).astype(np.float32) + g_h).astype(np.float32)
    for t in (x, u, z):
        assert np.array_equal(t.cpu().numpy(), want)
    assert np.array_equal(g.cpu().numpy(), g_h)


def test_stream_pattern_rejects_overlap():
    buf = torch.zeros(4 * 1024, dtype=torch.float32, device=DEV)
    with pytest.raises(sgp.SgpError):
        sgp.sgp_stream_pattern([buf[:2048]], [buf[1024:3072]])
