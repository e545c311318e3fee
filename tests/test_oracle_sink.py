"""Pins for the oracle's attention-sink tokens (paper Sec. 3.5: the first token(s) stay in fp16).
Everything here is checked against numpy formulas written independently of the oracle's C code."""
import numpy as np

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup

SCALE = 1.0 / np.sqrt(128.0)


def _numpy_scores(q, k16, n_kv_heads, base, scale):
    """Textbook attention scores of rotated queries against fp16 pre-RoPE keys, RoPE written with
    complex numbers: the pair (i, i+64) is k_i + 1j*k_{i+64}, rotated by exp(1j*n*theta_i)."""
    L, D = k16.shape
    Hq = q.shape[0]
    g = Hq // n_kv_heads
    theta = base ** (-2.0 * np.arange(64) / 128.0)
    k = k16.astype(np.float64).reshape(L, n_kv_heads, 128)
    z = (k[:, :, :64] + 1j * k[:, :, 64:]) * np.exp(1j * np.arange(L)[:, None, None] * theta[None, None, :])
    out = np.zeros((Hq, L))
    for h in range(Hq):
        qh = q[h].astype(np.float64)
        out[h] = scale * (z[:, h // g, :].real @ qh[:64] + z[:, h // g, :].imag @ qh[64:])
    return out


def _cache(st, cap, n_sink):
    wl = st.wl
    return O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                         st.s, st.z, st.lo, st.hi, n_sink=n_sink)


def test_all_tokens_kept_in_fp16_is_plain_fp16_attention():
    wl = S.workload("c4", n_kv_heads=2, n_q_heads=8)
    st = Setup(wl)
    L = 4
    k, v = st.k(0, L), st.v(0, L)
    oc = _cache(st, 128, n_sink=L)
    oc.append_k(k[:1]); oc.append_k(k[1:])          # chunks straddle nothing special: all rows are sinks
    oc.append_v(v[:3]); oc.append_v(v[3:])
    q = S.gen_q(wl, 0, 0)
    got = oc.qk(q, SCALE)
    ref = _numpy_scores(q, k, wl.n_kv_heads, wl.rope_base, SCALE)
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    p = O.softmax(got)
    ref_out = np.stack([p[h].astype(np.float64) @ v.astype(np.float64)[:, (h // 4) * 128:(h // 4 + 1) * 128]
                        for h in range(8)])
    assert np.allclose(oc.pv(p), ref_out, rtol=1e-6, atol=1e-7)


def test_one_sink_token_changes_only_its_own_terms():
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    L = 70
    k, v = st.k(0, L), st.v(0, L)
    a, b = _cache(st, 128, 0), _cache(st, 128, 1)
    for oc in (a, b):
        oc.append_k(k[:5]); oc.append_k(k[5:])
        oc.append_v(v)
    # the stored quantized cache does not depend on the sink setting
    for name in ("k_codes", "v_codes", "v_sz", "k_ptr", "v_ptr", "k_idx", "k_val", "v_idx", "v_val"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    assert np.array_equal(b.sink_k[0], k[0].view(np.uint16)) and np.array_equal(b.sink_v[0], v[0].view(np.uint16))
    q = S.gen_q(wl, 0, 0)
    sa, sb = a.qk(q, SCALE), b.qk(q, SCALE)
    assert np.array_equal(sa[:, 1:], sb[:, 1:])
    # position 0: RoPE is the identity there, so the score is a plain dot product with the fp16 key
    ref0 = np.array([SCALE * np.dot(q[h].astype(np.float64), k[0].astype(np.float64)[h * 128:(h + 1) * 128])
                     for h in range(4)])
    assert np.allclose(sb[:, 0], ref0, rtol=1e-6, atol=1e-6)
    assert not np.allclose(sa[:, 0], sb[:, 0], rtol=1e-9, atol=0)      # the quantized key differs from the fp16 one
    p = O.softmax(sb)
    oa, ob = a.pv(p).astype(np.float64), b.pv(p).astype(np.float64)
    vhat0 = a.reconstruct_v(0, 1)[0]
    delta = np.stack([p[h, 0] * (v[0].astype(np.float64) - vhat0)[h * 128:(h + 1) * 128] for h in range(4)])
    assert np.allclose(ob - oa, delta, rtol=1e-4, atol=2e-7)           # both outputs were rounded to fp32


def test_sink_rows_fill_across_append_chunks():
    wl = S.workload("c2", n_kv_heads=2, n_q_heads=2)
    st = Setup(wl)
    k, v = st.k(0, 9), st.v(0, 9)
    oc = _cache(st, 128, 3)
    for lo, hi in ((0, 2), (2, 7), (7, 9)):
        oc.append_k(k[lo:hi]); oc.append_v(v[lo:hi])
    assert np.array_equal(oc.sink_k, k[:3].view(np.uint16)) and np.array_equal(oc.sink_v, v[:3].view(np.uint16))
