"""Pins for the oracle's RoPE, score / output mat-vecs, softmax and storage accounting."""
import numpy as np
import pytest
import scipy.special

import kvq_synth as S
from oracle import kvq_oracle as O


def block_rope_matrix(d, n, base):
    """The block-diagonal rotation matrix of the paper's RoPE appendix (adjacent channel pairs
    (2i, 2i+1), theta_i = base^(-2i/d) with i counted from 0)."""
    R = np.zeros((d, d), dtype=np.longdouble)
    for i in range(d // 2):
        th = np.longdouble(base) ** (np.longdouble(-2.0 * i) / d)
        c, s = np.cos(n * th), np.sin(n * th)
        R[2 * i, 2 * i], R[2 * i, 2 * i + 1] = c, -s
        R[2 * i + 1, 2 * i], R[2 * i + 1, 2 * i + 1] = s, c
    return R


def half_split_perm(d):
    """perm[j] = position in the adjacent-pair ordering of half-split channel j."""
    p = np.zeros(d, dtype=int)
    for i in range(d // 2):
        p[i] = 2 * i
        p[i + d // 2] = 2 * i + 1
    return p


@pytest.mark.parametrize("n", [0, 1, 5, 4095, 131071, 1048575])
@pytest.mark.parametrize("base", [10000.0, 500000.0])
def test_rope_equals_block_matrix_under_channel_permutation(n, base):
    rng = np.random.default_rng(n % 1000)
    d = 128
    x = rng.standard_normal(d)
    y = O.rope(x, n, base)
    p = half_split_perm(d)
    xp = np.zeros(d, np.longdouble); xp[p] = x
    yp = block_rope_matrix(d, n, base) @ xp
    assert np.allclose(y, np.asarray(yp[p], dtype=np.float64), rtol=0, atol=1e-9)


def test_rope_identity_norm_and_unit_frequency():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(128)
    assert np.array_equal(O.rope(x, 0, 10000.0), x)
    for n in (3, 1000, 777777):
        y = O.rope(x, n, 10000.0)
        for i in range(64):     # each rotated pair keeps its length
            assert abs(np.hypot(y[i], y[i + 64]) - np.hypot(x[i], x[i + 64])) < 1e-12
        # theta_0 = 1: pair (0, 64) turns by exactly n radians
        assert abs(y[0] - (x[0] * np.cos(n) - x[64] * np.sin(n))) < 1e-9
        assert abs(y[64] - (x[64] * np.cos(n) + x[0] * np.sin(n))) < 1e-9


def test_rope_inner_product_depends_only_on_relative_position():
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal(128), rng.standard_normal(128)
    ref = O.rope(q, 50, 10000.0) @ O.rope(k, 20, 10000.0)
    for shift in (1, 1000, 100000):
        assert abs(O.rope(q, 50 + shift, 10000.0) @ O.rope(k, 20 + shift, 10000.0) - ref) < 1e-8


def numpy_rope_rows(K, base, n0=0):
    """Rotate rows of K [L][H*128] head by head with the block-matrix form (independent route)."""
    L, D = K.shape
    p = half_split_perm(128)
    out = np.zeros_like(K, dtype=np.float64)
    for n in range(L):
        R = np.asarray(block_rope_matrix(128, n0 + n, base), dtype=np.float64)
        for h in range(D // 128):
            xp = np.zeros(128); xp[p] = K[n, h * 128:(h + 1) * 128]
            out[n, h * 128:(h + 1) * 128] = (R @ xp)[p]
    return out


def exact_cache(bits, H, Hq, L, seed):
    """A cache whose quantisation is lossless: inputs are built from codes with power-of-two scales
    and signposts that are multiples of 2^-4, so dequantisation reproduces them exactly."""
    rng = np.random.default_rng(seed)
    D = H * 128
    n = 1 << bits
    lut = np.sort(rng.choice(np.arange(-16, 17), size=n, replace=False)).astype(np.float32) / 16
    lut[0], lut[-1] = -1.0, 1.0
    s_k = (2.0 ** rng.integers(-2, 3, D)).astype(np.float16)
    z_k = (rng.integers(-8, 9, D) / 4).astype(np.float16)
    big = np.full(D, 60000.0, np.float16)
    kc = rng.integers(0, n, (L, D))
    K = (s_k.astype(np.float64) * lut[kc] + z_k.astype(np.float64))
    s_v = 2.0 ** rng.integers(-2, 3, (L, 1))
    vc = rng.integers(1, n - 1, (L, D))
    vc[:, 0], vc[:, 1] = 0, n - 1                     # every token touches both ends of its range
    z_v = rng.integers(-8, 9, (L, 1)) / 4
    V = s_v * lut[vc] + z_v
    oc = O.OracleCache(bits, H, Hq, ((L + 127) // 128) * 128, 0, 10000.0, lut, lut, s_k, z_k, -big, big)
    ck = oc.append_k(K.astype(np.float16))
    cv = oc.append_v(V.astype(np.float16))
    assert np.array_equal(ck, kc) and np.array_equal(cv, vc)
    return oc, K, V


def test_softmax_subtracts_the_row_maximum():
    """Scores in the thousands: exp overflows even in double unless the maximum is subtracted first; the
    result must still be scipy's (which subtracts it) and every row must sum to 1.  A row of equal
    scores (uniform weights) rides along."""
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((3, 50)) * 900.0).astype(np.float32)
    x[1] = np.float32(-1234.5)
    p = O.softmax(x)
    assert np.all(np.isfinite(p))
    assert np.allclose(p, scipy.special.softmax(x.astype(np.float64), axis=1), rtol=1e-6, atol=1e-12)
    assert np.allclose(p.sum(1), 1.0, atol=1e-6)
    assert np.allclose(p[1], 1.0 / 50, rtol=1e-6)


@pytest.mark.parametrize("bits,H,Hq", [(3, 2, 2), (4, 1, 4), (2, 2, 8)])
def test_lossless_cache_reduces_to_textbook_attention_matvecs(bits, H, Hq):
    L = 200
    oc, K, V = exact_cache(bits, H, Hq, L, seed=bits)
    assert np.array_equal(oc.reconstruct_k(0, L), K)
    assert np.array_equal(oc.reconstruct_v(0, L), V)
    rng = np.random.default_rng(4)
    q = rng.standard_normal((Hq, 128)).astype(np.float32)
    scale = 1.0 / np.sqrt(128)
    Krot = numpy_rope_rows(K, 10000.0)
    g = Hq // H
    ref = np.stack([scale * (Krot[:, (h // g) * 128:(h // g + 1) * 128] @ q[h].astype(np.float64)) for h in range(Hq)])
    scores = oc.qk(q, scale)
    assert np.allclose(scores, ref, rtol=1e-6, atol=1e-6)
    probs = O.softmax(scores)
    assert np.allclose(probs, scipy.special.softmax(scores.astype(np.float64), axis=1), rtol=1e-6, atol=1e-9)
    assert np.allclose(probs.sum(1), 1.0, atol=1e-5)
    ref_out = np.stack([probs[h].astype(np.float64) @ V[:, (h // g) * 128:(h // g + 1) * 128] for h in range(Hq)])
    assert np.allclose(oc.pv(probs), ref_out, rtol=1e-6, atol=1e-6)


def test_sparse_part_equals_densified_outliers_and_rope_is_linear():
    """Dense + sparse through the oracle == textbook mat-vec on (dequantised + densified residuals)."""
    w = S.workload("c2", n_kv_heads=2, n_q_heads=4)
    L, bits = 256, 3
    lut_k, lut_v = S.make_lut(bits, w.seed, 0, 0), S.make_lut(bits, w.seed, 0, 1)
    s, z, lo, hi = S.calibrate_k(w)
    ks = S.k_side_from_fraction(0.01, w.D)
    oc = O.OracleCache(bits, 2, 4, L, ks, w.rope_base, lut_k, lut_v, s, z, lo, hi)
    ck = oc.append_k(S.gen_k(w, 0, 0, 0, L)); cv = oc.append_v(S.gen_v(w, 0, 0, 0, L))
    assert oc.k_ptr[L] > 0 and oc.v_ptr[L] == L * 2 * ks
    # a cache stores its signposts as fp16 numbers: the restatement below rounds them with numpy
    assert not np.array_equal(lut_k, lut_k.astype(np.float16).astype(np.float32))
    lut_k, lut_v = (a.astype(np.float16).astype(np.float32) for a in (lut_k, lut_v))
    sf, zf = s.astype(np.float32), z.astype(np.float32)
    Kd = (sf * lut_k[ck] + zf).astype(np.float64)
    Ksp = np.zeros_like(Kd)
    for n in range(L):
        for e in range(oc.k_ptr[n], oc.k_ptr[n + 1]):
            Ksp[n, oc.k_idx[e]] += np.float64(oc.k_val[e:e + 1].view(np.float16)[0])
    q = S.gen_q(w, 0, 0)
    ref = np.stack([(numpy_rope_rows(Kd, w.rope_base) + numpy_rope_rows(Ksp, w.rope_base))[:, (h // 2) * 128:(h // 2 + 1) * 128]
                    @ q[h].astype(np.float64) for h in range(4)]) * 0.25
    assert np.allclose(oc.qk(q, 0.25), ref, rtol=2e-6, atol=2e-5)
    svz = oc.v_sz.view(np.float16).astype(np.float32)
    Vd = (svz[:L, :1] * lut_v[cv] + svz[:L, 1:]).astype(np.float64)
    for n in range(L):
        for e in range(oc.v_ptr[n], oc.v_ptr[n + 1]):
            Vd[n, oc.v_idx[e]] += np.float64(oc.v_val[e:e + 1].view(np.float16)[0])
    p = O.softmax(oc.qk(q, 0.25))
    ref_out = np.stack([p[h].astype(np.float64) @ Vd[:, (h // 2) * 128:(h // 2 + 1) * 128] for h in range(4)])
    assert np.allclose(oc.pv(p), ref_out, rtol=2e-6, atol=2e-6)


def test_quantized_scores_track_the_unquantized_fp16_scores():
    """The whole chain (quantise, pack, dequantise, rotate, dot) stays close to plain fp16 attention."""
    w = S.workload("c2", n_kv_heads=2, n_q_heads=2)
    L, bits = 256, 4
    lut = np.linspace(-1, 1, 16).astype(np.float16).astype(np.float32)
    s, z, lo, hi = S.calibrate_k(w)
    oc = O.OracleCache(bits, 2, 2, L, S.k_side_from_fraction(0.01, w.D), w.rope_base, lut, lut, s, z, lo, hi)
    K = S.gen_k(w, 0, 0, 0, L); V = S.gen_v(w, 0, 0, 0, L)
    oc.append_k(K); oc.append_v(V)
    q = S.gen_q(w, 0, 0)
    Krot = numpy_rope_rows(K.astype(np.float64), w.rope_base)
    ref = np.stack([Krot[:, h * 128:(h + 1) * 128] @ q[h].astype(np.float64) for h in range(2)]) / np.sqrt(128)
    got = oc.qk(q, 1 / np.sqrt(128)).astype(np.float64)
    assert np.corrcoef(ref.ravel(), got.ravel())[0, 1] > 0.99
    p = O.softmax(ref.astype(np.float32))
    ref_out = np.stack([p[h].astype(np.float64) @ V[:, h * 128:(h + 1) * 128].astype(np.float64) for h in range(2)])
    assert np.corrcoef(ref_out.ravel(), oc.pv(p).astype(np.float64).ravel())[0, 1] > 0.99


def test_storage_accounting_matches_the_papers_average_bits_and_cache_sizes():
    """nuq3-1%: 3.32-3.35 bits/element; LLaMA-7B cache 64.0 -> 13.3 (128K) and 512 -> ~106.4 (1M)
    (paper: average-bit-width column of the perplexity tables; KV cache size table, App. on memory)."""
    H, d, layers = 32, 128, 32
    D = H * d
    for bits, lo_b, hi_b, gb128 in ((4, 4.32, 4.35, 17.3), (3, 3.32, 3.35, 13.3), (2, 2.32, 2.35, 9.3)):
        L = 131072
        ks = S.k_side_from_fraction(0.01, D)
        dense = O.codes_bytes(bits, H, L)
        assert dense * 8 == bits * L * D
        sparse = L * 2 * ks * 4 + (L + 1) * 4          # (idx16 + val16) per outlier, one 32-bit pointer per token
        k_bytes = dense + sparse                        # Keys: per-channel scale/zero are O(1) in L
        v_bytes = dense + sparse + L * 4                # Values: + fp16 scale and zero-point per token
        avg_bits = (k_bytes + v_bytes) * 8 / (2 * L * D)
        assert lo_b - 0.005 <= avg_bits <= hi_b + 0.005
        gib = layers * (k_bytes + v_bytes) / 2 ** 30
        assert abs(gib - gb128) < 0.06
        if bits == 3:
            assert abs(gib * 8 - 106.4) / 106.4 < 0.005     # 1M context = 8 x 128K
    assert 2 * layers * D * 2 * 131072 / 2 ** 30 == 64.0    # fp16 baseline, 2*n*h*d*e*b*l
