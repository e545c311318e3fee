"""Growth of FLAT sparse outlier arrays between appends (a larger allocation and a copy of the entries in
use, amortised by growing in steps): a cache that starts with room for a handful of outliers holds, bit for
bit, what a cache with the full capacity from the start holds, and the mat-vecs read it the same.  (Blocked
storage, which grows without copying, has its own test file.)"""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits,block", [(3, 256), (2, 1000), (4, 64)])
def test_flat_cache_grown_in_steps_equals_cache_with_full_capacity(bits, block):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=8, bits=bits)
    st = Setup(wl)
    L, cap, D = 700, 768, wl.D
    oc = st.oracle_cache(cap)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, cap_nnz_k=8, cap_nnz_v=8)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0, grown, caps = 0, 0, set()
    for i, T in enumerate([1, 1, 3, 64, 1, 200, 1, 130, 299]):
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        grown += gc.ensure_nnz_room(T * D, T * 2 * st.k_side, block=block)
        caps.add((gc.c.cap_nnz_k, gc.c.cap_nnz_v))
        assert all(c == 8 or c % block == 0 for c in (gc.c.cap_nnz_k, gc.c.cap_nnz_v))   # initial size or whole blocks
        if i % 2:
            K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        else:
            K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
            K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        t0 += T
    assert t0 == L and grown >= 3 and len(caps) >= 3           # several growth steps happened
    assert gc.status() == 0                                    # nothing was ever dropped
    assert not compare_caches(oc, gc)
    used_k, used_v = gc.nnz_used()
    assert used_k == int(oc.k_ptr[L]) and used_v == int(oc.v_ptr[L]) == L * 2 * st.k_side
    # the mat-vecs on the grown arrays
    q = S.gen_q(wl, 0, 0)
    scale = 1.0 / np.sqrt(128.0)
    scores = torch.zeros((wl.n_q_heads, cap), device="cuda")
    out = torch.zeros((wl.n_q_heads, 128), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), scale, scores, out)
    ref_scores = oc.qk(q, scale)
    ok, worst = matvec_close(scores.cpu().numpy()[:, :L], ref_scores)
    assert ok, f"scores: worst error / bound = {worst:.3f}"
    ok, worst = matvec_close(out.cpu().numpy(), oc.pv(O.softmax(ref_scores)), rel=2e-3)
    assert ok, f"outputs: worst error / bound = {worst:.3f}"


def test_without_growth_the_overflow_is_reported():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, 256, st.k_side, wl.rope_base, cap_nnz_k=8, cap_nnz_v=8)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    K.kvq_quantize_append_v(gc, torch.from_numpy(st.v(0, 40)).cuda())
    assert gc.status() == 4                                    # KVQ_ERR_NNZ_OVERFLOW
    assert gc.nnz_used()[1] == 8                               # pointers are clamped to the capacity
