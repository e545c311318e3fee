"""Pins of the calibration oracle (oracle/kvq_calib_oracle.py: the sensitivity-weighted k-means of
paper Sec. 3.3 Eq. (1) with the s_i^2 weighting of the appendix on per-channel scaling) against
things other than itself: the exact optimum by exhaustive search on tiny inputs, scikit-learn's
weighted Lloyd solver, closed forms, and invariances a wrong weight, index or update would break."""
import itertools

import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_calib_oracle as C


def _sse(x, w, groups):
    tot = 0.0
    for g in groups:
        if len(g) == 0:
            continue
        xs, ws = x[g].astype(np.float64), w[g].astype(np.float64)
        if ws.sum() == 0:
            continue
        m = np.sum(ws * xs) / ws.sum()
        tot += float(np.sum(ws * (xs - m) ** 2))
    return tot


def _exhaustive_optimum(x, w, k):
    """Minimum of the weighted 1-D k-means objective: an optimal partition of sorted points is made
    of contiguous runs, so all placements of k-1 cuts are tried."""
    order = np.argsort(x, kind="stable")
    n = x.size
    best, best_groups = None, None
    for cuts in itertools.combinations(range(1, n), k - 1):
        b = (0,) + cuts + (n,)
        groups = [order[b[i]:b[i + 1]] for i in range(k)]
        v = _sse(x, w, groups)
        if best is None or v < best:
            best, best_groups = v, groups
    return best, best_groups


def test_fixed_point_at_the_exhaustive_optimum_and_never_below_it():
    rng = np.random.default_rng(5)
    for trial in range(4):
        x = rng.uniform(-1, 1, 11).astype(np.float32)
        w = rng.lognormal(0, 1, 11).astype(np.float32)
        k = 4
        opt, groups = _exhaustive_optimum(x, w, k)
        c_opt = np.array([np.sum(w[g].astype(np.float64) * x[g]) / np.sum(w[g].astype(np.float64)) for g in groups],
                         dtype=np.float32)
        # started at the optimum the solver stays there and reports the optimal objective
        c = C.nuq_signposts(x, w, c_opt, 3)
        assert np.allclose(c, np.sort(c_opt), rtol=0, atol=1e-6)
        assert C.objective(x, w, c) == pytest.approx(opt, rel=1e-5, abs=1e-9)
        # from anywhere else it can only end at or above the optimum
        for _ in range(5):
            c0 = np.sort(rng.uniform(-1, 1, k)).astype(np.float32)
            assert C.objective(x, w, C.nuq_signposts(x, w, c0, 10)) >= opt - 1e-9


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_matches_sklearn_weighted_lloyd(bits):
    from sklearn.cluster import KMeans
    x, w = S.gen_calibration(20240118 + bits, 20000)
    k = 1 << bits
    c0 = np.linspace(-1, 1, k).astype(np.float32)
    iters = 7
    ours = C.nuq_signposts(x, w, c0, iters)
    km = KMeans(n_clusters=k, init=c0.reshape(-1, 1).astype(np.float64), n_init=1, max_iter=iters, tol=0.0,
                algorithm="lloyd").fit(x.reshape(-1, 1).astype(np.float64), sample_weight=w.astype(np.float64))
    theirs = np.sort(km.cluster_centers_.reshape(-1))
    assert km.n_iter_ == iters                     # not converged earlier: both made `iters` updates
    assert np.allclose(ours, theirs, rtol=2e-5, atol=2e-6)


def test_objective_never_increases_and_weights_matter():
    x, w = S.gen_calibration(7, 30000)
    c = np.linspace(-1, 1, 8).astype(np.float32)
    prev = C.objective(x, w, c)
    for _ in range(6):
        c = C.lloyd_step(x, w, c)
        cur = C.objective(x, w, c)
        assert cur <= prev * (1 + 1e-7)
        prev = cur
    # the sensitivity weights change the answer (a solver that dropped them would not notice): make the
    # right-hand part of the range ten times as sensitive and run both solvers to convergence
    xs, ws = x[:6000], (w[:6000] * np.where(x[:6000] > 0.3, np.float32(10.0), np.float32(1.0))).astype(np.float32)
    c_w = C.nuq_signposts(xs, ws, np.linspace(-1, 1, 8), 60)
    c_1 = C.nuq_signposts(xs, np.ones_like(ws), np.linspace(-1, 1, 8), 60)
    assert np.max(np.abs(c_w - c_1)) > 1e-2
    assert np.sum(c_w > 0.3) > np.sum(c_1 > 0.3)             # more signposts where the weight is
    assert C.objective(xs, ws, c_w) < C.objective(xs, ws, c_1)


def test_separated_groups_give_weighted_means():
    rng = np.random.default_rng(11)
    centres = np.array([-0.9, -0.3, 0.2, 0.8], dtype=np.float32)
    x = np.concatenate([c + rng.uniform(-0.02, 0.02, 50).astype(np.float32) for c in centres]).astype(np.float32)
    w = rng.lognormal(0, 1.5, x.size).astype(np.float32)
    got = C.nuq_signposts(x, w, centres + np.float32(0.05), 2)
    want = [np.average(x[i * 50:(i + 1) * 50].astype(np.float64), weights=w[i * 50:(i + 1) * 50].astype(np.float64))
            for i in range(4)]
    assert np.allclose(got, want, rtol=0, atol=1e-6)


def test_invariances_of_the_weights():
    x, w = S.gen_calibration(3, 5000)
    c0 = np.linspace(-1, 1, 8).astype(np.float32)
    base = C.nuq_signposts(x, w, c0, 5)
    # a common factor on all weights changes nothing (powers of two: exactly nothing)
    assert np.array_equal(C.nuq_signposts(x, w * np.float32(4.0), c0, 5), base)
    # an element of weight 2w is two elements of weight w
    x2 = np.concatenate([x, x[:1000]]); w2 = np.concatenate([w, w[:1000]])
    wd = w.copy(); wd[:1000] *= np.float32(2.0)
    assert np.allclose(C.nuq_signposts(x2, w2, c0, 5), C.nuq_signposts(x, wd, c0, 5), rtol=1e-6, atol=1e-7)
    # elements of weight zero do not exist for the solver, wherever they lie
    xz = np.concatenate([x, np.full(300, 0.77, np.float32)]); wz = np.concatenate([w, np.zeros(300, np.float32)])
    assert np.array_equal(C.nuq_signposts(xz, wz, c0, 5), base)
    # order of the elements is irrelevant up to fp64 summation order
    p = np.random.default_rng(0).permutation(x.size)
    assert np.allclose(C.nuq_signposts(x[p], w[p], c0, 5), base, rtol=1e-6, atol=1e-7)


def test_ties_go_to_the_smaller_index_and_empty_signposts_stay():
    c = np.array([-0.5, 0.0, 0.5, 0.9], dtype=np.float32)
    x = np.array([-0.25, 0.25, 0.7], dtype=np.float32)       # each exactly between two signposts
    assert list(C.nearest(x, c)) == [0, 1, 2]
    # signpost 3 gets nothing and keeps its place; the others move onto their single element
    out = C.lloyd_step(x, np.ones(3, np.float32), c)
    assert np.array_equal(out, np.array([-0.25, 0.25, 0.7, 0.9], dtype=np.float32))
    # a signpost whose elements all have weight zero stays too
    out = C.lloyd_step(x, np.array([1, 0, 1], np.float32), c)
    assert np.array_equal(out, np.array([-0.25, 0.0, 0.7, 0.9], dtype=np.float32))


def test_s_squared_weighting_is_the_unnormalised_error():
    """Appendix on per-channel scaling: with A = s*A_norm + z per channel, the Fisher-weighted error of A
    equals the error of A_norm weighted by F*s^2, for any set of signposts."""
    rng = np.random.default_rng(2)
    n_ch, n_tok = 6, 400
    s = rng.uniform(0.5, 4.0, n_ch); z = rng.uniform(-1, 1, n_ch)
    a_norm = rng.uniform(-1, 1, (n_tok, n_ch)).astype(np.float32)
    F = rng.lognormal(0, 1, (n_tok, n_ch))
    c = np.sort(rng.uniform(-1, 1, 8)).astype(np.float32)
    q_norm = c[C.nearest(a_norm.reshape(-1), c)].reshape(n_tok, n_ch).astype(np.float64)
    A = s * a_norm.astype(np.float64) + z
    QA = s * q_norm + z
    lhs = float(np.sum(F * (A - QA) ** 2))
    rhs = C.objective(a_norm.reshape(-1), (F * s ** 2).astype(np.float32).reshape(-1), c)
    assert rhs == pytest.approx(lhs, rel=1e-5)


def test_key_channel_constants_against_numpy_partition_and_counts():
    """Order statistics by np.partition (no sort), element counts on each side of the thresholds,
    and the mid-/half-range identities."""
    wl = S.workload("c2", n_kv_heads=2, n_q_heads=2)
    x = S.gen_k(wl, 0, 0, 0, 3000, tensor_id=7)
    p = 0.01
    s, z, lo, hi = C.key_channel_constants(x, p)
    T, D = x.shape
    k = 15                                                         # floor(0.005 * 3000 + 0.5)
    xf = x.astype(np.float32)
    part_lo = np.partition(xf, [k - 1, k], axis=0)
    part_hi = np.partition(xf, [T - k - 1, T - k], axis=0)
    assert np.array_equal(lo.astype(np.float32), part_lo[k - 1])
    assert np.array_equal(hi.astype(np.float32), part_hi[T - k])
    # at most k-1 elements lie strictly outside a threshold, at least k at or beyond it
    assert np.all((xf < lo.astype(np.float32)).sum(0) <= k - 1) and np.all((xf <= lo.astype(np.float32)).sum(0) >= k)
    assert np.all((xf > hi.astype(np.float32)).sum(0) <= k - 1) and np.all((xf >= hi.astype(np.float32)).sum(0) >= k)
    a, b = part_lo[k], part_hi[T - k - 1]
    assert np.array_equal(z, ((b + a) * np.float32(0.5)).astype(np.float16))
    sc = ((b - a) * np.float32(0.5)).astype(np.float16)
    assert np.array_equal(s, np.where(sc.astype(np.float32) > 0, sc, np.float16(1.0)))
    # every inlier normalises into [-1, 1] up to the fp16 rounding of scale and zero-point
    inl = (xf >= a) & (xf <= b)
    xn = (xf - z.astype(np.float32)) / s.astype(np.float32)
    assert np.max(np.abs(xn[inl])) <= 1.0 + 2e-3


@pytest.mark.parametrize("fraction", [0.01, 0.01006, 0.0012])
def test_key_channel_constants_equal_the_input_generators_calibration(fraction):
    """The synthetic-input package calibrates its Key channels with code of its own (numpy, written
    for input generation): same data, same constants.  The fractions put fraction/2 * 4096 at 20.48,
    20.60 and 2.46: rounding the outlier count to the nearest integer matters for the second."""
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4, outlier_fraction=fraction)
    prof = S.key_channel_profile(wl, 0)
    from kvq_synth.gen import T_KCAL
    x = S.gen_k(wl, 0, 0, 0, 4096, profile=prof, tensor_id=T_KCAL)
    s, z, lo, hi = C.key_channel_constants(x, wl.outlier_fraction)
    gs, gz, glo, ghi = S.calibrate_k(wl, 0, n_cal=4096, profile=prof)
    for a, b in ((s, gs), (z, gz), (lo, glo), (hi, ghi)):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_key_channel_constants_degenerate_cases():
    x = np.zeros((64, 3), np.float16)
    x[:, 1] = np.arange(64, dtype=np.float16)                      # 0..63
    x[:, 2] = np.float16(2.5)                                      # constant channel
    s, z, lo, hi = C.key_channel_constants(x, 0.0)                 # no outliers: open thresholds, full range
    assert np.all(lo == np.float16(-65504)) and np.all(hi == np.float16(65504))
    assert z[1] == np.float16(31.5) and s[1] == np.float16(31.5)
    assert s[0] == np.float16(1.0) and z[0] == np.float16(0.0) and s[2] == np.float16(1.0) and z[2] == np.float16(2.5)
    s, z, lo, hi = C.key_channel_constants(x, 2.0 / 64 * 2)        # k = 2 per side
    assert lo[1] == np.float16(1.0) and hi[1] == np.float16(62.0)
    assert z[1] == np.float16(31.5) and s[1] == np.float16(29.5)   # range [2, 61]
    assert lo[2] == np.float16(2.5) and hi[2] == np.float16(2.5) and s[2] == np.float16(1.0)
