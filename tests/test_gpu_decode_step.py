"""The one-call generation step (append the new token's Key and Value, then the fused attention over the
cache that ends with it; paper Sec. 3): what kvq_quantize_append_kv followed by kvq_attention_decode
gives - bit for bit where the step runs those two calls, to 2e-5 of a row's RMS where its first launch
holds the append and the sparse Key kernel together (the same terms summed over other sub-ranges of
tokens) -, the cache bit for bit the oracle's, the outputs within the chained tolerance of the oracle's
qk -> softmax -> pv (twice the mat-vec tolerance: a score error delta multiplies a weight by e^delta),
and a rejected call changes nothing."""
import ctypes as C

import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


@pytest.mark.parametrize("name,bits,kvh,qh,n_sink,blocked", [
    ("c2", 3, 8, 8, 0, False),          # D = 1024: append and sparse Key kernel in one launch
    ("c2", 3, 32, 32, 0, False),        # D = 4096, the bench shape: likewise, sixteen wavefronts on the Value
    ("c4", 2, 8, 32, 2, False),         # grouped heads, sink tokens, from an empty cache
    ("c3", 4, 32, 32, 0, False),
    ("c4", 2, 4, 16, 2, False),         # D = 512: the two calls
    ("c3", 4, 8, 8, 0, True)])          # blocked storage: the two calls
def test_decode_step_equals_append_then_attention(name, bits, kvh, qh, n_sink, blocked):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload(name, n_kv_heads=kvh, n_q_heads=qh, bits=bits, outlier_fraction=0.01)
    st = Setup(wl)
    cap, L0, steps = 1280, 1100, 40
    oc = O.OracleCache(wl.bits, kvh, qh, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi,
                       cap_nnz_k=st.cap_nnz_k(cap), n_sink=n_sink)
    kw = dict(nnz_block_entries=1024) if blocked else {}
    a, b = (K.KvqCache(wl.bits, kvh, qh, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap), n_sink=n_sink, **kw)
            for _ in range(2))
    for c in (a, b):
        K.kvq_lut_load(c, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    if n_sink:                                   # sinks arrive through the step call too: start from nothing
        L0 = 0
    else:
        k, v = st.k(0, L0), st.v(0, L0)
        oc.append_k(k); oc.append_v(v)
        for c in (a, b):
            K.kvq_quantize_append_kv(c, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
    one_launch = not blocked and wl.D in (1024, 4096)
    assert K.kvq_decode_step_launches(a) == (5 if one_launch else 6) + (1 if n_sink else 0)
    sa, sb = (torch.zeros((qh, cap), device="cuda") for _ in range(2))
    oa, ob = (torch.zeros((qh, 128), device="cuda") for _ in range(2))
    for i in range(steps):
        t = L0 + i
        k, v, q = st.k(t, 1), st.v(t, 1), S.gen_q(wl, 0, 0, step=i)
        kd, vd, qd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(q).cuda()
        K.kvq_decode_step(a, kd, vd, qd, SCALE, sa, oa)
        K.kvq_quantize_append_kv(b, kd, vd)
        K.kvq_attention_decode(b, qd, SCALE, sb, ob)
        assert a.n_tokens_k == a.n_tokens_v == t + 1
        if not one_launch:
            assert torch.equal(sa, sb) and torch.equal(oa, ob)
        else:
            ok, worst = matvec_close(sa.cpu().numpy()[:, :t + 1], sb.cpu().numpy()[:, :t + 1], rel=2e-5)
            assert ok, f"step {i}: scores against the two calls, worst error / bound = {worst:.3f}"
            ok, worst = matvec_close(oa.cpu().numpy(), ob.cpu().numpy(), rel=2e-5)
            assert ok, f"step {i}: outputs against the two calls, worst error / bound = {worst:.3f}"
        oc.append_k(k); oc.append_v(v)
        if i % 13 == 0 or i == steps - 1:
            ref = oc.qk(q, SCALE)
            ok, worst = matvec_close(sa.cpu().numpy()[:, :t + 1], ref)
            assert ok, f"step {i}: scores worst error / bound = {worst:.3f}"
            ok, worst = matvec_close(oa.cpu().numpy(), oc.pv(O.softmax(ref)), rel=2e-3)
            assert ok, f"step {i}: outputs worst error / bound = {worst:.3f}"
    assert a.status() == 0 and not compare_caches(oc, a)


def test_a_rejected_step_changes_nothing():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    gc = st.gpu_cache(256)
    lib = K.load_library()
    k, v = torch.from_numpy(st.k(0, 1)).cuda(), torch.from_numpy(st.v(0, 1)).cuda()
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores, out = torch.zeros((4, 256), device="cuda"), torch.zeros((4, 128), device="cuda")
    K.kvq_quantize_append_kv(gc, torch.from_numpy(st.k(0, 9)).cuda(), torch.from_numpy(st.v(0, 9)).cuda())
    before = [t.clone() for t in (gc.k_codes, gc.v_codes, gc.k_ptr, gc.v_ptr)]

    def call(k_=k, v_=v, q_=q, ld=256, sc=scores, o=out):
        p = lambda t: t.data_ptr() if t is not None else None
        return lib.kvq_decode_step(C.byref(gc.c), p(k_), p(v_), p(q_), C.c_float(0.1), p(sc), ld, p(o), None)

    assert call(ld=9) == 1                       # no room for the new token's score
    assert call(q_=None) == 1 and call(sc=None) == 1 and call(o=None) == 1 and call(k_=None) == 1 and call(v_=None) == 1
    ws, gc.c.workspace_bytes = gc.c.workspace_bytes, 1024
    assert call() == 3                           # workspace too small for the attention half
    gc.c.workspace_bytes = ws
    gc.c.n_tokens_v -= 1
    assert call() == 1                           # Keys and Values out of step
    gc.c.n_tokens_v += 1
    torch.cuda.synchronize()
    assert gc.n_tokens_k == 9 and gc.n_tokens_v == 9
    assert all(torch.equal(x, y) for x, y in zip(before, (gc.k_codes, gc.v_codes, gc.k_ptr, gc.v_ptr)))
    assert call() == 0 and gc.n_tokens_k == 10


def test_step_with_full_outlier_arrays_reports_overflow_like_the_two_calls():
    """The step's first launch on a cache whose Key outlier array fills up during the step: the sticky
    status is set, pointers are clamped, and scores and outputs are those of the two calls on a twin
    (which drops the same entries)."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    cap, L0 = 128, 100
    a, b = (K.KvqCache(wl.bits, 8, 8, cap, st.k_side, wl.rope_base, cap_nnz_k=16 * cap) for _ in range(2))
    for c in (a, b):
        K.kvq_lut_load(c, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
        K.kvq_quantize_append_kv(c, torch.from_numpy(st.k(0, L0)).cuda(), torch.from_numpy(st.v(0, L0)).cuda())
    assert K.kvq_decode_step_launches(a) == 5 and a.status() == 0
    hi, lo = (np.asarray(x, dtype=np.float16).astype(np.float32) for x in (st.hi, st.lo))
    full = (hi + 4.0 * (hi - lo) + 1.0).astype(np.float16)[None, :]          # every channel an outlier
    sa, sb = (torch.zeros((8, cap), device="cuda") for _ in range(2))
    oa, ob = (torch.zeros((8, 128), device="cuda") for _ in range(2))
    for i in range(3):                                                     # 3 x 1024 entries: the array overflows
        kd, vd = torch.from_numpy(full).cuda(), torch.from_numpy(st.v(L0 + i, 1)).cuda()
        qd = torch.from_numpy(S.gen_q(wl, 0, 0, step=i)).cuda()
        K.kvq_decode_step(a, kd, vd, qd, SCALE, sa, oa)
        K.kvq_quantize_append_kv(b, kd, vd)
        K.kvq_attention_decode(b, qd, SCALE, sb, ob)
        n = L0 + i + 1
        ok, worst = matvec_close(sa.cpu().numpy()[:, :n], sb.cpu().numpy()[:, :n], rel=2e-5)
        assert ok, f"step {i}: scores worst error / bound = {worst:.3f}"
        ok, worst = matvec_close(oa.cpu().numpy(), ob.cpu().numpy(), rel=2e-5)
        assert ok, f"step {i}: outputs worst error / bound = {worst:.3f}"
    assert a.status() == 4 and b.status() == 4
    assert torch.equal(a.k_ptr, b.k_ptr) and int(a.k_ptr[L0 + 3].item()) == 16 * cap
    assert torch.equal(a.k_idx, b.k_idx) and torch.equal(a.k_val, b.k_val) and torch.equal(a.k_codes, b.k_codes)
