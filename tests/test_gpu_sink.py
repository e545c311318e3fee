"""GPU parity for attention-sink tokens (paper Sec. 3.5: the first tokens stay in fp16): the HIP path
against the oracle, whose sink semantics are pinned to numpy attention in test_oracle_sink.py."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


def _pair(st, cap, n_sink, L, chunks):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=st.cap_nnz_k(cap), n_sink=n_sink)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap),
                    n_sink=n_sink)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0, i = 0, 0
    while t0 < L:
        T = min(chunks[i % len(chunks)], L - t0)
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        t0 += T
        i += 1
    torch.cuda.synchronize()
    return oc, gc


def _check(st, oc, gc, L, n_sink):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    ns = min(n_sink, L)
    D = wl.D
    assert np.array_equal(gc.sink_k.cpu().numpy().view(np.uint16)[:ns * D], oc.sink_k[:ns].reshape(-1))
    assert np.array_equal(gc.sink_v.cpu().numpy().view(np.uint16)[:ns * D], oc.sink_v[:ns].reshape(-1))
    q = S.gen_q(wl, 0, 0)
    ref = oc.qk(q, SCALE)
    scores = torch.full((wl.n_q_heads, L + 2), 5.0, device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
    got = scores.cpu().numpy()
    assert np.all(got[:, L:] == 5.0)
    ok, worst = matvec_close(got[:, :L], ref)
    assert ok, f"qk worst error / bound = {worst:.3f}"
    # the sink columns themselves, against their own magnitude (fp16 keys: fp32 arithmetic error only)
    assert np.allclose(got[:, :ns], ref[:, :ns], rtol=1e-4, atol=1e-4)
    for temp in (1.0, 0.02):                     # the second distribution puts most weight on few tokens
        logits = ref / temp
        p = O.softmax(logits.astype(np.float32))
        p[:, 0] = np.maximum(p[:, 0], 0.05)      # make sure the first sink token carries weight
        p = (p / p.sum(1, keepdims=True)).astype(np.float32)
        out = torch.empty((wl.n_q_heads, 128), device="cuda")
        K.kvq_pv_matvec(gc, torch.from_numpy(p).cuda(), out)
        ok, worst = matvec_close(out.cpu().numpy(), oc.pv(p))
        assert ok, f"pv worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("name,ov,n_sink,L,chunks", [
    ("c2", dict(n_kv_heads=8, n_q_heads=8), 1, 300, [1, 2, 130]),
    ("c4", dict(n_kv_heads=2, n_q_heads=8), 3, 200, [2, 64]),       # the second chunk straddles the sink boundary
    ("c3", dict(n_kv_heads=4, n_q_heads=4, outlier_fraction=0.004), 4, 131, [131]),
    ("c2", dict(n_kv_heads=4, n_q_heads=4), 4, 3, [1]),             # fewer tokens than sinks: all in fp16
    ("c2", dict(n_kv_heads=4, n_q_heads=4, outlier_fraction=0.0), 2, 129, [5]),   # no outliers at all
])
def test_sink_tokens_match_oracle(name, ov, n_sink, L, chunks):
    wl = S.workload(name, **ov)
    st = Setup(wl)
    oc, gc = _pair(st, 384, n_sink, L, chunks)
    _check(st, oc, gc, L, n_sink)


def test_sink_changes_result_and_bad_count_is_rejected():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4, bits=2)       # 2-bit: the sink matters most
    st = Setup(wl)
    _, g0 = _pair(st, 128, 0, 64, [64])
    _, g1 = _pair(st, 128, 1, 64, [64])
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    s0, s1 = torch.zeros((4, 64), device="cuda"), torch.zeros((4, 64), device="cuda")
    K.kvq_qk_matvec(g0, q, SCALE, s0)
    K.kvq_qk_matvec(g1, q, SCALE, s1)
    assert torch.equal(s0[:, 1:], s1[:, 1:]) and not torch.equal(s0[:, 0], s1[:, 0])
    g1.c.n_sink = 5
    with pytest.raises(K.KvqError):
        K.kvq_qk_matvec(g1, q, SCALE, s1)
    g1.c.n_sink = 1
    g1.c.sink_v = 0
    with pytest.raises(K.KvqError):
        K.kvq_pv_matvec(g1, s1, torch.zeros((4, 128), device="cuda"))
