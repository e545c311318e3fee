"""GPU softmax helper against the oracle's (which is pinned to scipy): both load paths (rows aligned
to 16 bytes or not), ragged lengths around the chunk and vector sizes, extreme dynamic range."""
import numpy as np
import pytest

from oracle import kvq_oracle as O

pytestmark = pytest.mark.gpu


def _run(x, ld, offset):
    """x: [H, n] float32.  The device matrix has row stride `ld` and starts `offset` floats into an
    aligned allocation (offset 0 and ld % 4 == 0 take the 16-byte path)."""
    import torch
    import paper_2401_18079_amd as K
    H, n = x.shape
    buf = torch.full((H * ld + offset + 8,), 77.0, device="cuda")
    xin = buf[offset:offset + H * ld].view(H, ld)
    xin[:, :n] = torch.from_numpy(x).cuda()
    obuf = torch.full((H * ld + offset + 8,), -5.0, device="cuda")
    out = obuf[offset:offset + H * ld].view(H, ld)
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(H, n), dtype=torch.uint8, device="cuda")
    K.kvq_softmax_f32(xin, out, n, ws)
    got = out.cpu().numpy()
    assert np.all(got[:, n:] == -5.0)                        # padding columns untouched
    assert np.all(obuf.cpu().numpy()[:offset] == -5.0)
    return got[:, :n]


@pytest.mark.parametrize("n", [1, 3, 4, 255, 4096, 4097, 9001, 20000])
@pytest.mark.parametrize("ld_extra,offset", [(0, 0), (4, 0), (3, 0), (4, 1), (0, 2)])
def test_softmax_matches_oracle(n, ld_extra, offset):
    rng = np.random.default_rng(n * 31 + ld_extra * 7 + offset)
    x = (rng.standard_normal((5, n)) * 3).astype(np.float32)
    ld = n + ld_extra
    if ld_extra == 4:
        ld = (n + 3) // 4 * 4 + 4                            # a multiple of four: the 16-byte path when offset is 0
    got = _run(x, ld, offset)
    ref = O.softmax(x)
    assert np.allclose(got, ref, rtol=2e-5, atol=1e-9)
    assert np.allclose(got.sum(1), 1.0, atol=1e-4)


def test_softmax_extreme_rows():
    n = 10000
    rng = np.random.default_rng(3)
    x = np.zeros((6, n), dtype=np.float32)
    x[0] = rng.uniform(-1e4, 1e4, n)                          # one element takes everything
    x[1] = 123.456                                            # constant row: uniform distribution
    x[2] = -3.0e38                                            # at the float range's lower end
    x[2, 77] = -2.9e38
    x[3] = rng.standard_normal(n) * 1e-3
    x[4, :] = -80.0; x[4, 5000] = 80.0
    x[5] = np.linspace(-50, 50, n)
    for ld, off in ((n, 0), (n + 3, 1)):
        got = _run(x, ld, off)
        ref = O.softmax(x)
        assert np.all(np.isfinite(got))
        assert np.allclose(got, ref, rtol=3e-5, atol=1e-12)
        assert np.allclose(got.sum(1), 1.0, atol=1e-4)
