"""GPU parity for the combined append (Keys and Values of the same tokens in one call, one launch for
the quantization): the cache it builds must be bit-identical to the oracle's, whose append is the
paper's online quantization (Sec. 3.1-3.4, 3.6) step by step."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches

pytestmark = pytest.mark.gpu


def _caches(st, cap, n_sink=0):
    import paper_2401_18079_amd as K
    wl = st.wl
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=st.cap_nnz_k(cap), n_sink=n_sink)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap),
                    n_sink=n_sink)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    return oc, gc


@pytest.mark.parametrize("name,ov,n_sink,chunks", [
    ("c2", dict(n_kv_heads=32, n_q_heads=32), 0, [1, 1, 1, 130, 1, 64, 1]),      # the bench shape (D = 4096)
    ("c2", dict(n_kv_heads=16, n_q_heads=16), 0, [1, 520, 1, 511]),               # D = 2048: bulk and wide-workgroup calls
    ("c2", dict(n_kv_heads=8, n_q_heads=8, bits=2), 0, [1, 5, 1, 200]),
    ("c3", dict(n_kv_heads=8, n_q_heads=8, outlier_fraction=0.004), 0, [3, 1, 1, 77]),
    ("c4", dict(n_kv_heads=2, n_q_heads=8), 0, [1, 1, 300, 1]),                  # D = 256: the 256-thread kernels
    ("c2", dict(n_kv_heads=12, n_q_heads=12), 0, [1, 65, 1]),                    # D = 1536: ragged last pass
    ("c2", dict(n_kv_heads=8, n_q_heads=8), 3, [1, 1, 2, 60]),                   # attention-sink rows copied too
    ("c2", dict(n_kv_heads=4, n_q_heads=4, outlier_fraction=0.0), 0, [1, 40, 1]),
    ("c2", dict(n_kv_heads=96, n_q_heads=96), 0, [1, 2, 40, 1]),                 # D = 12288: three passes of 4096 channels
    ("c2", dict(n_kv_heads=128, n_q_heads=128, bits=4), 0, [1, 30]),             # D = 16384: the widest Value append
])
def test_append_kv_bit_exact(name, ov, n_sink, chunks):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload(name, **ov)
    st = Setup(wl)
    L = sum(chunks)
    cap = (L + 127) // 128 * 128 + 128
    oc, gc = _caches(st, cap, n_sink)
    t0 = 0
    for T in chunks:
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        t0 += T
        assert gc.n_tokens_k == t0 and gc.n_tokens_v == t0
    torch.cuda.synchronize()
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    if n_sink:
        D = wl.D
        assert np.array_equal(gc.sink_k.cpu().numpy().view(np.uint16)[:n_sink * D], oc.sink_k[:n_sink].reshape(-1))
        assert np.array_equal(gc.sink_v.cpu().numpy().view(np.uint16)[:n_sink * D], oc.sink_v[:n_sink].reshape(-1))


def test_append_kv_mixes_with_separate_appends_and_unequal_counts():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    oc, gc = _caches(st, 512)
    # Keys run two tokens ahead of Values, then both advance together
    k = st.k(0, 2); oc.append_k(k); K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    nk, nv = 2, 0
    for T in (1, 1, 33, 1):
        k, v = st.k(nk, T), st.v(nv, T)
        oc.append_k(k); oc.append_v(v)
        K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        nk += T; nv += T
    v = st.v(nv, 2); oc.append_v(v); K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
    torch.cuda.synchronize()
    assert gc.n_tokens_k == 38 and gc.n_tokens_v == 38
    assert gc.status() == 0
    assert not compare_caches(oc, gc)


def test_appends_from_inputs_that_are_only_2_byte_aligned():
    """New-token matrices that start one fp16 element into an allocation: legal for every append call
    (the boundary asks for fp16 alignment only), so no kernel may rely on wider loads of them."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    oc, gc = _caches(st, 512)

    def shifted(a):
        buf = torch.zeros(a.size + 1, dtype=torch.float16, device="cuda")
        buf[1:] = torch.from_numpy(a).cuda().reshape(-1)
        x = buf[1:].view(a.shape)
        assert x.data_ptr() % 16 == 2 and x.is_contiguous()
        return x

    t0 = 0
    for T, combined in ((1, True), (37, True), (1, False), (90, False)):
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        if combined:
            K.kvq_quantize_append_kv(gc, shifted(k), shifted(v))
        else:
            K.kvq_quantize_append_k(gc, shifted(k))
            K.kvq_quantize_append_v(gc, shifted(v))
        t0 += T
    torch.cuda.synchronize()
    assert gc.status() == 0
    assert not compare_caches(oc, gc)


def test_value_appends_wider_than_16384_channels_are_refused():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=136, n_q_heads=136)         # D = 17408
    st = Setup(wl)
    gc = st.gpu_cache(128)
    k, v = torch.from_numpy(st.k(0, 2)).cuda(), torch.from_numpy(st.v(0, 2)).cuda()
    for call in (lambda: K.kvq_quantize_append_kv(gc, k, v), lambda: K.kvq_quantize_append_v(gc, v)):
        with pytest.raises(K.KvqError) as e:
            call()
        assert e.value.status == 2                               # KVQ_ERR_UNSUPPORTED, nothing launched
    assert gc.n_tokens_k == 0 and gc.n_tokens_v == 0
    oc = st.oracle_cache(128)
    oc.append_k(st.k(0, 2))
    K.kvq_quantize_append_k(gc, k)                               # Keys alone have no such limit
    torch.cuda.synchronize()
    assert gc.status() == 0 and np.array_equal(gc.k_codes.cpu().numpy(), oc.k_codes)
    nk = int(oc.k_ptr[2])
    assert np.array_equal(gc.k_idx.cpu().numpy().view(np.uint16)[:nk], oc.k_idx[:nk])


def test_append_kv_overflow_and_argument_errors():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    gc = st.gpu_cache(128)
    k, v = torch.from_numpy(st.k(0, 4)).cuda(), torch.from_numpy(st.v(0, 4)).cuda()
    with pytest.raises(AssertionError):
        K.kvq_quantize_append_kv(gc, k, v[:3])                   # the binding insists on equal token counts
    K.kvq_quantize_append_kv(gc, k, v)
    big_k = torch.from_numpy(st.k(4, 125)).cuda()
    big_v = torch.from_numpy(st.v(4, 125)).cuda()
    with pytest.raises(K.KvqError):                              # 4 + 125 > capacity 128: nothing is appended
        K.kvq_quantize_append_kv(gc, big_k, big_v)
    assert gc.n_tokens_k == 4 and gc.n_tokens_v == 4
    gc.c.k_side_v = wl.D                                         # more outliers than elements
    with pytest.raises(K.KvqError):
        K.kvq_quantize_append_kv(gc, k, v)
    assert gc.n_tokens_k == 4 and gc.n_tokens_v == 4

    # sparse arrays too small: the sticky device status reports it and the dense codes stay valid,
    # exactly as for the separate calls
    g2 = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, 128, st.k_side, wl.rope_base, cap_nnz_k=16, cap_nnz_v=16)
    K.kvq_lut_load(g2, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    oc = st.oracle_cache(128)
    for t0, T in ((0, 1), (1, 1), (2, 38)):
        kk, vv = st.k(t0, T), st.v(t0, T)
        oc.append_k(kk); oc.append_v(vv)
        K.kvq_quantize_append_kv(g2, torch.from_numpy(kk).cuda(), torch.from_numpy(vv).cuda())
    torch.cuda.synchronize()
    assert g2.status() == 4
    assert np.array_equal(g2.k_codes.cpu().numpy(), oc.k_codes)
    assert np.array_equal(g2.v_codes.cpu().numpy(), oc.v_codes)
    kp = g2.k_ptr.cpu().numpy().view(np.uint32)
    assert kp.max() <= 16 and np.all(np.diff(kp[:41].astype(np.int64)) >= 0)
    assert np.array_equal(g2.k_idx.cpu().numpy().view(np.uint16)[:16], oc.k_idx[:16])
