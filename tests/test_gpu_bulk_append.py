"""Bulk appends (calls of a thousand tokens and more take the wavefront-per-token Key kernel, calls
of 512 and more the four-wavefronts-per-token Value kernel where the layer has one of the widths it
is built for, 1024 to 8192 channels): bit-exact against the oracle for every code width, head counts
that fill no workgroup evenly, calls that are not a multiple of the four tokens a workgroup takes,
sink rows, tokens full of equal elements, and a bulk call that overflows the sparse arrays."""
import numpy as np
import pytest

import kvq_synth as S
from kvq_testlib import Setup, compare_caches

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,ov,n_sink,chunks", [
    ("c2", dict(n_kv_heads=3, n_q_heads=3), 0, [1025, 1, 1500]),                 # D = 384
    ("c2", dict(n_kv_heads=8, n_q_heads=8, bits=2), 2, [1024, 1027]),
    ("c3", dict(n_kv_heads=4, n_q_heads=8, outlier_fraction=0.004), 0, [2049]),  # 4-bit
    ("c4", dict(n_kv_heads=1, n_q_heads=4), 1, [1100, 1100]),                    # one head: two channels per lane in all
    ("c2", dict(n_kv_heads=4, n_q_heads=4, outlier_fraction=0.0), 0, [1300]),    # thresholds admit no outlier
    ("c2", dict(n_kv_heads=16, n_q_heads=16), 0, [513, 600]),                    # D = 2048
    ("c3", dict(outlier_fraction=0.004), 1, [601]),                              # D = 4096, 4-bit
    ("c2", dict(bits=2), 0, [512]),                                              # D = 4096, 2-bit
    ("c2", dict(n_kv_heads=40, n_q_heads=40), 1, [513]),                         # D = 5120
    ("c3", dict(n_kv_heads=52, n_q_heads=52, outlier_fraction=0.004), 0, [1, 512]),   # D = 6656, 4-bit, odd start
    ("c2", dict(n_kv_heads=64, n_q_heads=64, bits=2), 0, [600]),                 # D = 8192
])
def test_bulk_appends_bit_exact(name, ov, n_sink, chunks):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload(name, **ov)
    st = Setup(wl)
    L = sum(chunks)
    cap = (L + 127) // 128 * 128 + 128
    from oracle import kvq_oracle as O
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=st.cap_nnz_k(cap), n_sink=n_sink)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap),
                    n_sink=n_sink)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0 = 0
    for i, T in enumerate(chunks):
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        if i % 2:
            K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
            K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        else:
            K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        t0 += T
    torch.cuda.synchronize()
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    if n_sink:
        D = wl.D
        assert np.array_equal(gc.sink_k.cpu().numpy().view(np.uint16)[:n_sink * D], oc.sink_k[:n_sink].reshape(-1))


def test_bulk_key_append_that_overflows_the_sparse_array():
    """1200 tokens into room for 3000 Key outliers: the pointers stop at the capacity, the entries that
    fit are the oracle's first 3000, the status word reports the overflow, the packed codes are whole."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    T, cap, room = 1200, 1280, 3000
    oc = st.oracle_cache(cap)
    gc = K.KvqCache(wl.bits, 4, 4, cap, st.k_side, wl.rope_base, cap_nnz_k=room)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    k = st.k(0, T)
    oc.append_k(k)
    assert int(oc.k_ptr[T]) > room                              # the case is what it claims to be
    K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    torch.cuda.synchronize()
    assert gc.status() == 4                                     # KVQ_ERR_NNZ_OVERFLOW
    assert np.array_equal(gc.k_codes.cpu().numpy(), oc.k_codes)
    kp = gc.k_ptr.cpu().numpy().view(np.uint32)[:T + 1]
    assert np.array_equal(kp, np.minimum(oc.k_ptr[:T + 1], room))
    assert np.array_equal(gc.k_idx.cpu().numpy().view(np.uint16)[:room], oc.k_idx[:room])
    assert np.array_equal(gc.k_val.cpu().numpy().view(np.uint16)[:room], oc.k_val[:room])


@pytest.mark.parametrize("heads,bits", [(8, 3), (16, 4), (32, 3), (32, 2), (40, 3), (64, 4)])
def test_bulk_value_append_ties(heads, bits):
    """Bulk Value appends of vectors full of equal elements: ties at one or both thresholds, thresholds
    that coincide, all elements equal.  The choice among equal elements must be the oracle's (lower
    channel first, the upper side before the lower one) wherever the tied channels fall among the
    wavefronts that share a token."""
    import torch
    import paper_2401_18079_amd as K
    from kvq_testlib import tie_vectors
    wl = S.workload("c2", n_kv_heads=heads, n_q_heads=heads, bits=bits)
    st = Setup(wl)
    assert st.k_side >= 1
    rng = np.random.default_rng(300 + heads)
    rows = tie_vectors(wl.D, st.k_side, rng)
    T = 530                                                     # one bulk call, from an odd token on
    v = np.stack([np.roll(rows[i % len(rows)], 37 * i) for i in range(T)])
    v[1::3] = v[1::3, ::-1]
    lead = st.v(0, 1)
    k = st.k(0, T + 1)
    oc, gc = st.oracle_cache(640), st.gpu_cache(640)
    oc.append_k(k); oc.append_v(lead); oc.append_v(v)
    K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    K.kvq_quantize_append_v(gc, torch.from_numpy(lead).cuda())
    K.kvq_quantize_append_v(gc, torch.from_numpy(np.ascontiguousarray(v)).cuda())
    torch.cuda.synchronize()
    assert gc.status() == 0
    bad = compare_caches(oc, gc)
    assert not bad, bad
