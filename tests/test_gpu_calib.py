"""GPU parity for the offline datatype derivation (kvq_calibrate_nuq: the sensitivity-weighted k-means
of paper Sec. 3.3 Eq. (1)) against the CPU oracle, which tests/test_oracle_calib.py pins.

Tolerance.  Both sides decide the assignment from the same fp32 distances and round a signpost to
fp32 after every update; only the order of the fp64 additions differs, which changes a sum by ~1e-16
of itself and so, rarely, the last fp32 bit of a signpost.  A signpost that differs by one fp32 ulp can
move an element that sits within an ulp of the boundary between two signposts to the other side; with
n elements per signpost that shifts a mean by ~1/n of the gap.  The bound below, 2e-6 absolute on
signposts in [-1, 1], is a few fp32 ulps and far above all of that for the sizes tested."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_calib_oracle as C

pytestmark = pytest.mark.gpu

ATOL = 2e-6


def _gpu(x, w, bits, iters, init):
    import torch
    import paper_2401_18079_amd as K
    return K.kvq_calibrate_nuq(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), bits, iters, init)


@pytest.mark.parametrize("bits,n,iters", [
    (2, 300003, 5),          # several hundred workgroups and a ragged tail of three elements
    (3, 300003, 5),
    (4, 300003, 5),
    (3, 1 << 20, 12),
    (4, 4097, 9),
    (3, 1024, 4),            # exactly one group of four per lane of one workgroup
    (2, 5, 3), (3, 3, 2), (4, 1, 1),   # fewer elements than signposts, tail-only inputs
])
def test_signposts_match_oracle(bits, n, iters):
    x, w = S.gen_calibration(20240118 + 10 * bits, n)
    c0 = np.linspace(-1, 1, 1 << bits).astype(np.float32)
    got = _gpu(x, w, bits, iters, c0)
    ref = C.nuq_signposts(x, w, c0, iters)
    assert got.dtype == np.float32 and np.all(np.diff(got) >= 0)
    assert np.allclose(got, ref, rtol=0, atol=ATOL), (got, ref)


def test_every_iteration_matches_the_oracle_step_by_step():
    x, w = S.gen_calibration(99, 200001)
    c = np.linspace(-1, 1, 8).astype(np.float32)
    for it in range(6):
        nxt = _gpu(x, w, 3, 1, c)
        assert np.allclose(nxt, np.sort(C.lloyd_step(x, w, c)), rtol=0, atol=ATOL), it
        c = nxt


def test_empty_and_weightless_signposts_unsorted_start_and_zero_iterations():
    x, w = S.gen_calibration(5, 50000)
    # a signpost far outside the data attracts nothing and stays; the start need not be sorted
    c0 = np.array([0.3, 5.0, -0.4, -0.9, 0.0, 0.8, -7.0, 0.5], dtype=np.float32)
    got = _gpu(x, w, 3, 4, c0)
    ref = C.nuq_signposts(x, w, c0, 4)
    assert got[0] == -7.0 and got[-1] == 5.0
    assert np.allclose(got, ref, rtol=0, atol=ATOL)
    # all weight zero near one signpost: it stays as well
    w2 = np.where(np.abs(x - 0.5) < 0.12, np.float32(0.0), w).astype(np.float32)
    c1 = np.array([-0.8, -0.4, -0.1, 0.1, 0.3, 0.5, 0.7, 0.9], dtype=np.float32)
    got = _gpu(x, w2, 3, 1, c1)
    assert 0.5 in got
    assert np.allclose(got, C.nuq_signposts(x, w2, c1, 1), rtol=0, atol=ATOL)
    # no iteration: the start, sorted
    assert np.array_equal(_gpu(x, w, 3, 0, c0), np.sort(c0))


def test_ties_go_to_the_smaller_index_on_the_gpu_too():
    c = np.array([-0.5, 0.0, 0.5, 0.9], dtype=np.float32)
    x = np.array([-0.25, 0.25, 0.7, 0.7, -0.25], dtype=np.float32)     # all exactly between two signposts
    w = np.array([1, 2, 3, 1, 1], dtype=np.float32)
    got = _gpu(x, w, 2, 1, c)
    assert np.array_equal(got, C.nuq_signposts(x, w, c, 1))
    assert np.array_equal(got, np.array([-0.25, 0.25, 0.7, 0.9], dtype=np.float32))


def test_large_input_in_the_launch_configuration_of_a_real_layer():
    """8M elements (a 2K-token calibration sample of a 4096-channel layer), 4-bit: the grid is capped
    and every lane walks many groups."""
    n = (1 << 23) + 1
    x, w = S.gen_calibration(77, n)
    c0 = np.linspace(-1, 1, 16).astype(np.float32)
    got = _gpu(x, w, 4, 3, c0)
    assert np.allclose(got, C.nuq_signposts(x, w, c0, 3), rtol=0, atol=ATOL)


def test_argument_errors():
    import torch
    import paper_2401_18079_amd as K
    x = torch.zeros(1024, device="cuda"); w = torch.ones(1024, device="cuda")
    with pytest.raises(K.KvqError):
        K.kvq_calibrate_nuq(x[1:], w[1:], 3, 1, np.linspace(-1, 1, 8))          # not 16-byte aligned
    with pytest.raises(AssertionError):
        K.kvq_calibrate_nuq(x, w, 3, 1, np.linspace(-1, 1, 4))                  # wrong number of signposts
    lib = K.load_library()
    ws = torch.zeros(int(lib.kvq_calibrate_workspace_bytes()), dtype=torch.uint8, device="cuda")
    c = np.linspace(-1, 1, 32).astype(np.float32)
    import ctypes
    p = c.ctypes.data_as(ctypes.c_void_p)
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert lib.kvq_calibrate_nuq(x.data_ptr(), w.data_ptr(), 1024, 5, 1, p, ws.data_ptr(), ws.numel(), sp) != 0   # bits
    assert lib.kvq_calibrate_nuq(x.data_ptr(), w.data_ptr(), 0, 3, 1, p, ws.data_ptr(), ws.numel(), sp) != 0      # n
    assert lib.kvq_calibrate_nuq(x.data_ptr(), w.data_ptr(), 1024, 3, -1, p, ws.data_ptr(), ws.numel(), sp) != 0  # iters
    assert lib.kvq_calibrate_nuq(x.data_ptr(), w.data_ptr(), 1024, 3, 1, p, ws.data_ptr(), 1000, sp) != 0         # workspace


# ---- per-channel Key calibration (thresholds, scale, zero-point): bit-exact against the oracle ----------

def _gpu_channels(x16, p):
    import torch
    import paper_2401_18079_amd as K
    return K.kvq_calibrate_key_channels(torch.from_numpy(x16).cuda(), p)


def _same(got, ref):
    for name, a, b in zip(("s", "z", "lo", "hi"), got, ref):
        a, b = np.asarray(a).view(np.uint16), np.asarray(b).view(np.uint16)
        assert np.array_equal(a, b), (name, int(np.sum(a != b)), np.nonzero(a != b)[0][:5])


@pytest.mark.parametrize("heads,T,p", [
    (4, 4096, 0.01),
    (4, 3000, 0.01),          # T not a multiple of the workgroup size
    (4, 4096, 0.01006),       # fraction/2 * T = 20.6: the outlier count rounds to the nearest integer, 21
    (4, 100, 0.05),           # fraction/2 * T = 2.5: a half rounds up, 3
    (32, 4096, 0.01),         # the bench layer's width
    (2, 32768, 0.001),        # the largest calibration set (16 samples of 2K tokens)
    (2, 700, 0.0),            # no outliers: open thresholds, full range
    (2, 65, 0.4),             # a quarter of every channel on each side
    (1, 1, 0.0),              # a single calibration token
])
def test_key_channel_constants_match_oracle(heads, T, p):
    wl = S.workload("c2", n_kv_heads=heads, n_q_heads=heads)
    from kvq_synth.gen import T_KCAL
    x = S.gen_k(wl, 0, 0, 0, T, tensor_id=T_KCAL)
    _same(_gpu_channels(x, p), C.key_channel_constants(x, p))


def test_key_channel_constants_with_heavy_ties_and_special_values():
    rng = np.random.default_rng(3)
    T, D = 2048, 256
    x = rng.integers(-3, 4, size=(T, D)).astype(np.float16)            # seven distinct values: ties everywhere
    x[:, 0] = np.float16(1.25)                                         # a constant channel
    x[:, 1] = np.where(rng.random(T) < 0.5, np.float16(0.0), np.float16(-0.0))   # +0 and -0 only
    x[:, 2] = rng.standard_normal(T).astype(np.float16) * np.float16(1e-6)       # subnormals
    x[:5, 3] = np.float16(65504.0); x[5:10, 3] = np.float16(-65504.0)            # the largest finite values
    for p in (0.01, 0.05, 0.0):
        _same(_gpu_channels(x, p), C.key_channel_constants(x, p))


def test_calibrated_constants_feed_the_cache():
    """End to end: constants calibrated on the GPU load into a cache and the append matches the oracle
    run with the oracle-calibrated constants."""
    import torch
    import paper_2401_18079_amd as K
    from oracle import kvq_oracle as O
    from kvq_synth.gen import T_KCAL
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    prof = S.key_channel_profile(wl, 0)
    xcal = S.gen_k(wl, 0, 0, 0, 4096, profile=prof, tensor_id=T_KCAL)
    s, z, lo, hi = _gpu_channels(xcal, wl.outlier_fraction)
    lut_k, lut_v = S.make_lut(wl.bits, wl.seed, 0, 0), S.make_lut(wl.bits, wl.seed, 0, 1)
    k_side = S.k_side_from_fraction(wl.outlier_fraction, wl.D)
    gc = K.KvqCache(wl.bits, 4, 4, 256, k_side, wl.rope_base, 64 * 256)
    K.kvq_lut_load(gc, lut_k, lut_v, s, z, lo, hi)
    rs, rz, rlo, rhi = C.key_channel_constants(xcal, wl.outlier_fraction)
    oc = O.OracleCache(wl.bits, 4, 4, 256, k_side, wl.rope_base, lut_k, lut_v, rs, rz, rlo, rhi, cap_nnz_k=64 * 256)
    k = S.gen_k(wl, 0, 0, 0, 200, profile=prof)
    oc.append_k(k)
    K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    torch.cuda.synchronize()
    assert gc.status() == 0
    assert np.array_equal(gc.k_codes.cpu().numpy(), oc.k_codes)
    nk = int(oc.k_ptr[200])
    assert np.array_equal(gc.k_idx.cpu().numpy().view(np.uint16)[:nk], oc.k_idx[:nk])
    assert 0.005 < nk / (200 * wl.D) < 0.02                        # about the calibrated 1 % are outliers


def test_key_channel_calibration_argument_errors():
    import torch
    import paper_2401_18079_amd as K
    x = torch.zeros((64, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(K.KvqError):
        K.kvq_calibrate_key_channels(x, 1.0)                           # 2k >= T
    with pytest.raises(K.KvqError):
        K.kvq_calibrate_key_channels(x, -0.1)
    big = torch.zeros((32769, 2), dtype=torch.float16, device="cuda")
    with pytest.raises(K.KvqError):
        K.kvq_calibrate_key_channels(big, 0.01)                        # more tokens than a channel's LDS holds
