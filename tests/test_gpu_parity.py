"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, fill_both, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)

# (workload overrides, context, append chunk pattern): several 64/128-token tiles plus a ragged tail
CASES = [
    ("c1", dict(), 1000, [1, 3, 64, 200]),
    ("c2", dict(n_kv_heads=8, n_q_heads=8), 777, [1, 2, 130, 64]),
    ("c2", dict(n_kv_heads=32, n_q_heads=32), 300, [300]),
    ("c3", dict(n_kv_heads=8, n_q_heads=8, outlier_fraction=0.004), 515, [64, 1]),
    ("c4", dict(), 450, [7, 128]),
    ("c4", dict(bits=3, n_kv_heads=2, n_q_heads=16), 259, [259]),
    ("c2", dict(bits=2, n_kv_heads=4, n_q_heads=8, outlier_fraction=0.0), 200, [33]),
]


def _ids(c):
    name, ov, L, ch = c
    return f"{name}-{'-'.join(f'{k}{v}' for k, v in ov.items())}-L{L}"


@pytest.fixture(scope="module", params=CASES, ids=_ids)
def pair(request):
    import torch
    name, ov, L, chunks = request.param
    wl = S.workload(name, **ov)
    st = Setup(wl)
    cap = ((L + 130 + 127) // 128) * 128
    oc, gc = st.oracle_cache(cap), st.gpu_cache(cap)
    fill_both(st, oc, gc, L, chunks)
    torch.cuda.synchronize()
    return st, oc, gc, L


def test_append_is_bit_exact(pair):
    st, oc, gc, L = pair
    assert gc.n_tokens_k == L and gc.n_tokens_v == L and gc.status() == 0
    bad = compare_caches(oc, gc)
    assert not bad, bad


def test_qk_scores_match_oracle(pair):
    import torch
    import paper_2401_18079_amd as K
    st, oc, gc, L = pair
    q = S.gen_q(st.wl, 0, 0)
    ref = oc.qk(q, SCALE)
    scores = torch.full((st.wl.n_q_heads, L + 5), 123.0, device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
    got = scores.cpu().numpy()
    assert np.all(got[:, L:] == 123.0)                 # entries past n_tokens are untouched
    ok, worst = matvec_close(got[:, :L], ref)
    assert ok, f"worst error / bound = {worst:.3f}"


def test_softmax_and_pv_match_oracle(pair):
    import torch
    import paper_2401_18079_amd as K
    st, oc, gc, L = pair
    q = S.gen_q(st.wl, 0, 0)
    ref_scores = oc.qk(q, SCALE)
    ref_p = O.softmax(ref_scores)
    x = torch.from_numpy(ref_scores).cuda()
    p = torch.empty_like(x)
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(x.shape[0], L), dtype=torch.uint8, device="cuda")
    K.kvq_softmax_f32(x, p, L, ws)
    gp = p.cpu().numpy()
    assert np.allclose(gp, ref_p, rtol=1e-4, atol=1e-9)
    assert np.allclose(gp.sum(1), 1.0, atol=1e-4)
    ref_out = oc.pv(ref_p)
    out = torch.empty((st.wl.n_q_heads, 128), device="cuda")
    K.kvq_pv_matvec(gc, torch.from_numpy(ref_p).cuda(), out)
    ok, worst = matvec_close(out.cpu().numpy(), ref_out)
    assert ok, f"worst error / bound = {worst:.3f}"
    # a peaked distribution (one dominant token) exercises the small-weight end
    logits = S.gen_probs_logits(st.wl, 0, 0, L, temperature=6.0)
    pp = O.softmax(logits)
    ref2 = oc.pv(pp)
    K.kvq_pv_matvec(gc, torch.from_numpy(pp).cuda(), out)
    ok, worst = matvec_close(out.cpu().numpy(), ref2)
    assert ok, f"peaked: worst error / bound = {worst:.3f}"


def test_decode_step_sequence_matches_oracle():
    """Append one token then attend, repeatedly, across a 64/128-token block boundary."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    oc, gc = st.oracle_cache(384), st.gpu_cache(384)
    fill_both(st, oc, gc, 120, [120])
    out = torch.empty((8, 128), device="cuda")
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(8, 384), dtype=torch.uint8, device="cuda")
    for step in range(12):
        n = 120 + step
        k, v = st.k(n, 1), st.v(n, 1)
        oc.append_k(k); oc.append_v(v)
        K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        q = S.gen_q(wl, 0, 0, step=step)
        scores = torch.zeros((8, 384), device="cuda")
        K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
        probs = torch.zeros_like(scores)
        K.kvq_softmax_f32(scores, probs, n + 1, ws)
        K.kvq_pv_matvec(gc, probs, out)
        rs = oc.qk(q, SCALE)
        rp = O.softmax(rs)
        ro = oc.pv(rp)
        ok, worst = matvec_close(scores.cpu().numpy()[:, :n + 1], rs)
        assert ok, (step, worst)
        ok, worst = matvec_close(out.cpu().numpy(), ro, rel=2e-3)   # probs come from GPU scores here
        assert ok, (step, worst)
    assert not compare_caches(oc, gc)


def test_edge_cases_and_error_codes():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=2, n_q_heads=2)
    st = Setup(wl)
    gc = st.gpu_cache(128)
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores = torch.full((2, 8), 7.0, device="cuda")
    out = torch.full((2, 128), 7.0, device="cuda")
    K.kvq_qk_matvec(gc, q, SCALE, scores)                     # empty cache: nothing written
    K.kvq_pv_matvec(gc, scores, out)                          # empty cache: zeros
    torch.cuda.synchronize()
    assert torch.all(scores == 7.0) and torch.all(out == 0.0)
    # a single token
    oc = st.oracle_cache(128)
    fill_both(st, oc, gc, 1, [1])
    K.kvq_qk_matvec(gc, q, SCALE, scores)
    ref = oc.qk(q.cpu().numpy(), SCALE)
    assert matvec_close(scores.cpu().numpy()[:, :1], ref)[0]
    # capacity: 128 tokens fit, the 129th does not
    fill_both(st, oc, gc, 127, [127])   # note: fill_both appends tokens [0,127) again as new tokens
    assert gc.n_tokens_k == 128
    with pytest.raises(K.KvqError) as e:
        K.kvq_quantize_append_k(gc, torch.from_numpy(st.k(0, 1)).cuda())
    assert e.value.status == 3 and gc.n_tokens_k == 128
    with pytest.raises(K.KvqError):
        K.kvq_quantize_append_v(gc, torch.from_numpy(st.v(0, 2)).cuda())
    # unsupported / invalid descriptors are rejected on the host
    bad = st.gpu_cache(128)
    bad.c.bits = 5
    with pytest.raises(K.KvqError) as e:
        K.kvq_qk_matvec(bad, q, SCALE, scores)
    assert e.value.status == 2
    notloaded = K.KvqCache(3, 2, 2, 128, st.k_side, 10000.0, 1024)
    with pytest.raises(K.KvqError) as e:
        K.kvq_quantize_append_k(notloaded, torch.from_numpy(st.k(0, 1)).cuda())
    assert e.value.status == 5


def test_sparse_overflow_sets_status_and_keeps_dense_codes():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    import paper_2401_18079_amd as K
    gc = K.KvqCache(wl.bits, 4, 4, 128, st.k_side, wl.rope_base, cap_nnz_k=16, cap_nnz_v=16)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    oc = st.oracle_cache(128)
    k, v = st.k(0, 40), st.v(0, 40)
    oc.append_k(k); oc.append_v(v)
    K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
    torch.cuda.synchronize()
    assert gc.status() == 4
    assert np.array_equal(gc.k_codes.cpu().numpy(), oc.k_codes)
    assert np.array_equal(gc.v_codes.cpu().numpy(), oc.v_codes)
    kp = gc.k_ptr.cpu().numpy().view(np.uint32)
    assert kp.max() <= 16 and np.all(np.diff(kp[:41].astype(np.int64)) >= 0)
    assert np.array_equal(gc.k_idx.cpu().numpy().view(np.uint16)[:16], oc.k_idx[:16])


def test_fp16_baselines_match_torch():
    import torch
    import paper_2401_18079_amd as K
    torch.manual_seed(0)
    for Hkv, Hq, L in ((32, 32, 1000), (8, 32, 333)):
        k16 = torch.randn(L, Hkv * 128, device="cuda", dtype=torch.float16)
        v16 = torch.randn(L, Hkv * 128, device="cuda", dtype=torch.float16)
        q = torch.randn(Hq, 128, device="cuda")
        r = Hq // Hkv
        scores = torch.zeros(Hq, L, device="cuda")
        K.kvq_fp16_qk_matvec(k16, Hkv, Hq, q, SCALE, scores)
        kk = k16.float().view(L, Hkv, 128).repeat_interleave(r, dim=1)        # [L][Hq][128]
        ref = torch.einsum("lhc,hc->hl", kk, q) * SCALE
        assert torch.allclose(scores, ref, rtol=1e-4, atol=1e-4)
        p = torch.softmax(ref, dim=1)
        out = torch.zeros(Hq, 128, device="cuda")
        ws = torch.zeros(K.binding.kvq_fp16_pv_workspace_bytes(Hq, L), dtype=torch.uint8, device="cuda")
        K.kvq_fp16_pv_matvec(v16, Hkv, Hq, p, out, ws)
        vv = v16.float().view(L, Hkv, 128).repeat_interleave(r, dim=1)
        ref_o = torch.einsum("hl,lhc->hc", p, vv)
        assert torch.allclose(out, ref_o, rtol=1e-4, atol=1e-5)


def test_device_generator_equals_host_generator():
    import torch
    from kvq_synth.device import DeviceGen
    for name, ov in (("c2", dict(n_kv_heads=4, n_q_heads=4)), ("c1", dict())):
        wl = S.workload(name, **ov)
        st = Setup(wl)
        dg = DeviceGen(wl, 0, st.kprof, st.vprof)
        for t0, T in ((0, 64), (100000, 33)):
            assert np.array_equal(dg.k(t0, T).cpu().numpy().view(np.uint16), st.k(t0, T).view(np.uint16))
            assert np.array_equal(dg.v(t0, T).cpu().numpy().view(np.uint16), st.v(t0, T).view(np.uint16))
