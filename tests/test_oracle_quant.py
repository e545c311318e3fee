"""Pins for the oracle's quantisation (nearest signpost, Key per-channel, Value per-token)."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O


def uniform_lut(bits):
    n = 1 << bits
    return (-1.0 + 2.0 * np.arange(n) / (n - 1)).astype(np.float32)


def f16(x):
    return np.asarray(x, dtype=np.float32).astype(np.float16)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_nearest_equals_sorted_midpoint_search_and_is_a_true_argmin(bits):
    rng = np.random.default_rng(bits)
    lut = S.make_lut(bits, 99, 0, 0)
    mids = (lut[:-1].astype(np.float64) + lut[1:].astype(np.float64)) / 2
    xs = rng.uniform(-1.3, 1.3, 4000).astype(np.float32)
    xs = xs[np.min(np.abs(xs[:, None].astype(np.float64) - mids[None, :]), axis=1) > 1e-6]
    for x in xs:
        j = O.nearest(lut, x)
        assert j == int(np.searchsorted(mids, float(x)))            # independent method
        d = np.abs(np.float32(x) - lut)
        assert d[j] == d.min()                                       # invariant
    # exact ties resolve to the smaller index
    lut2 = np.array([-1.0, -0.5, 0.5, 1.0], np.float32)
    assert O.nearest(lut2, 0.0) == 1
    assert O.nearest(lut2, -0.75) == 0
    assert O.nearest(lut2, 0.75) == 2


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_value_quant_with_uniform_lut_and_no_outliers_is_plain_minmax_uniform(bits):
    """Textbook special case: asymmetric min-max uniform quantisation (the intX baseline)."""
    rng = np.random.default_rng(11 + bits)
    T, D = 8, 256
    x = f16(rng.standard_normal((T, D)) * rng.uniform(0.5, 4, (T, 1)))
    lut = uniform_lut(bits)
    sz, codes, cnt, idx, val = O.quantize_v(x, bits, lut, 0)
    assert cnt.sum() == 0 and idx.size == 0
    xf = x.astype(np.float64)
    mn, mx = xf.min(1, keepdims=True), xf.max(1, keepdims=True)
    levels = (1 << bits) - 1
    u = (xf - mn) / (mx - mn) * levels
    ref = np.rint(u)
    safe = np.abs(u - np.floor(u) - 0.5) > 2e-2     # away from rounding ties (s,z are fp16-rounded)
    assert safe.mean() > 0.9
    assert np.array_equal(codes[safe].astype(np.float64), ref[safe])
    # scale / zero-point are the fp16-rounded half-range / mid-range
    assert np.array_equal(sz[:, 0], f16((mx - mn)[:, 0] * 0.5).view(np.uint16))
    assert np.array_equal(sz[:, 1], f16((mx + mn)[:, 0] * 0.5).view(np.uint16))


def test_key_quant_matches_numpy_restatement_and_threshold_rule():
    """Per-channel Keys: strict thresholds, residual = fp16(x - fp32 dequant)."""
    rng = np.random.default_rng(5)
    T, D, bits = 16, 256, 3
    lut = S.make_lut(bits, 5, 0, 0)
    s = f16(rng.uniform(0.5, 3, D)); z = f16(rng.standard_normal(D))
    lo = f16(z.astype(np.float32) - 1.5 * s.astype(np.float32)); hi = f16(z.astype(np.float32) + 1.5 * s.astype(np.float32))
    x = f16(rng.standard_normal((T, D)) * 2 * s.astype(np.float32) + z.astype(np.float32))
    x[0, 0] = lo[0]; x[0, 1] = hi[1]                      # exactly on a threshold: NOT an outlier
    codes, cnt, idx, val = O.quantize_k(x, bits, lut, s, z, lo, hi)
    xf, sf, zf = x.astype(np.float32), s.astype(np.float32), z.astype(np.float32)
    is_out = (xf < lo.astype(np.float32)) | (xf > hi.astype(np.float32))
    assert not is_out[0, 0] and not is_out[0, 1]
    assert np.array_equal(cnt, is_out.sum(1).astype(np.uint32))
    tt, cc = np.nonzero(is_out)                           # row-major: token, ascending channel
    assert np.array_equal(idx, cc.astype(np.uint16))
    xn = (xf - zf) * (np.float32(1.0) / sf)
    ref_codes = np.argmin(np.abs(xn[..., None] - lut), axis=-1)
    assert np.array_equal(codes, ref_codes.astype(np.uint8))
    deq = (sf.astype(np.float64) * lut[codes].astype(np.float64) + zf.astype(np.float64)).astype(np.float32)
    resid = f16(xf[tt, cc] - deq[tt, cc]).view(np.uint16)
    assert np.array_equal(val, resid)


def brute_topk(xrow, k):
    """Outlier set by full sort with the stated tie rules, written independently with lexsort."""
    D = xrow.size
    idx = np.arange(D)
    order_desc = np.lexsort((idx, -xrow))
    upper = order_desc[:k]
    rest = np.setdiff1d(idx, upper)
    order_asc = rest[np.lexsort((rest, xrow[rest]))]
    lower = order_asc[:k]
    return np.sort(np.concatenate([upper, lower]))


@pytest.mark.parametrize("D,k", [(128, 1), (1024, 5), (4096, 20), (4096, 2)])
def test_value_topk_against_full_sort_with_ties(D, k):
    rng = np.random.default_rng(D + k)
    T, bits = 6, 3
    x = f16(rng.standard_normal((T, D)) * 2)
    x[1] = f16(np.round(x[1].astype(np.float32)))          # heavy ties everywhere
    x[2, :] = np.float16(0.5)                              # all equal
    x[2, 7] = np.float16(-0.0); x[2, 9] = np.float16(0.0)
    x[3, : 4 * k] = np.float16(9.0)                        # more tied maxima than k
    x[4, -4 * k:] = np.float16(-9.0)
    lut = S.make_lut(bits, 1, 0, 1)
    sz, codes, cnt, idx, val = O.quantize_v(x, bits, lut, k)
    assert np.all(cnt == 2 * k)
    for t in range(T):
        got = idx[t * 2 * k:(t + 1) * 2 * k].astype(np.int64)
        assert np.all(np.diff(got) > 0)                    # ascending, no duplicates
        xr = x[t].astype(np.float32)
        assert np.array_equal(got, brute_topk(xr, k))
        keep = np.ones(D, bool); keep[got] = False
        s, z = sz[t].view(np.float16).astype(np.float32)
        mx, mn = xr[keep].max(), xr[keep].min()
        assert xr[got].max() >= mx and xr[got].min() <= mn
        zz = f16((mx + mn) * np.float32(0.5)); ss = f16((mx - mn) * np.float32(0.5))
        assert z == zz.astype(np.float32)
        assert s == (ss.astype(np.float32) if ss != 0 else np.float32(1.0))


def test_value_topk_rejects_too_many_outliers():
    x = f16(np.zeros((1, 128)))
    with pytest.raises(ValueError):
        O.quantize_v(x, 3, uniform_lut(3), 64)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_error_bound_for_non_outliers_and_exact_outliers(bits):
    """Non-outliers are within s*(largest signpost gap)/2 (+fp16 slack); outliers are
    reproduced to fp16 rounding of the residual by dense + sparse."""
    w = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    lut = S.make_lut(bits, w.seed, 0, 1)
    k = S.k_side_from_fraction(0.01, w.D)
    x = S.gen_v(w, 0, 0, 0, 32)
    sz, codes, cnt, idx, val = O.quantize_v(x, bits, lut, k)
    s = sz[:, 0].view(np.float16).astype(np.float64)[:, None]
    z = sz[:, 1].view(np.float16).astype(np.float64)[:, None]
    deq = (s.astype(np.float32) * lut[codes] + z.astype(np.float32)).astype(np.float64)  # approx of fmaf
    xf = x.astype(np.float64)
    is_out = np.zeros(x.shape, bool)
    tt = np.repeat(np.arange(32), 2 * k)
    is_out[tt, idx] = True
    gaps = np.diff(np.concatenate([[-1.0], lut.astype(np.float64), [1.0]]))
    bound = s * gaps.max() / 2 + (np.abs(z) + s) * 2.0 ** -10
    assert np.all(np.abs(xf - deq)[~is_out] <= np.broadcast_to(bound, x.shape)[~is_out])
    resid = val.view(np.float16).astype(np.float64)
    err = np.abs(deq[tt, idx] + resid - xf[tt, idx])
    assert np.all(err <= np.abs(resid) * 2.0 ** -11 + 2.0 ** -24 + np.abs(deq[tt, idx]) * 2.0 ** -22)


def test_nearly_everything_sparse_reproduces_fp16_input():
    """With k_side = D/2-1 all but two elements are outliers: reconstruction == input to fp16 rounding."""
    w = S.workload("c1")
    x = S.gen_v(w, 0, 0, 0, 128)
    lut = S.make_lut(3, w.seed, 0, 1)
    oc = O.OracleCache(3, 1, 1, 128, 63, 10000.0, lut, lut, *([np.ones(128, np.float16)] * 2 + [-np.ones(128, np.float16) * 60000] + [np.ones(128, np.float16) * 60000]))
    oc.append_v(x)
    vh = oc.reconstruct_v(0, 128)
    xf = x.astype(np.float64)
    assert np.all(np.abs(vh - xf) <= np.abs(xf) * 2.0 ** -10 + 1e-3)
    assert np.median(np.abs(vh - xf)) < 1e-3
