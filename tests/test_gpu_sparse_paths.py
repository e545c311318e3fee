"""GPU parity for the sparse (outlier) kernels on inputs chosen to reach every branch of them:
tokens without any Key outlier, a token whose channels are all outliers, outlier counts large enough
that a sub-range of tokens needs several batches of entries, and sparse arrays with no slack after
the last entry (loads near the end must not run past the arrays)."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


def _crafted_keys(st, L, rng):
    """Synthetic keys with planted rows: empty rows sit at the channels' mid-points (inside every
    threshold), full rows far outside them."""
    k = st.k(0, L).copy()
    z, hi, lo = (np.asarray(a, dtype=np.float16).astype(np.float32) for a in (st.z, st.hi, st.lo))
    empty = rng.choice(L, size=L // 5, replace=False)
    k[empty] = z.astype(np.float16)
    # runs of consecutive empty tokens, including the very first and the very last token
    k[0:3] = z.astype(np.float16)
    k[L - 2:L] = z.astype(np.float16)
    k[40:59] = z.astype(np.float16)
    full = [7, 64, L // 2]
    sign = np.where(rng.random(st.wl.D) < 0.5, -1.0, 1.0).astype(np.float32)
    far = np.where(sign > 0, hi + 4.0 * (hi - lo) + 1.0, lo - 4.0 * (hi - lo) - 1.0)
    k[full] = far.astype(np.float16)
    return k, empty, full


def _run(st, k, v, L, cap, cap_nnz_k=None, cap_nnz_v=None, chunks=(1, 5, 64, 130)):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=cap_nnz_k or wl.D * cap,
                       cap_nnz_v=cap_nnz_v or max(1, 2 * st.k_side * cap))
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base,
                    cap_nnz_k or wl.D * cap, cap_nnz_v=cap_nnz_v or max(1, 2 * st.k_side * cap))
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0, i = 0, 0
    while t0 < L:
        T = min(chunks[i % len(chunks)], L - t0)
        oc.append_k(k[t0:t0 + T]); oc.append_v(v[t0:t0 + T])
        K.kvq_quantize_append_k(gc, torch.from_numpy(k[t0:t0 + T]).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v[t0:t0 + T]).cuda())
        t0 += T
        i += 1
    torch.cuda.synchronize()
    return oc, gc


def _check_matvecs(st, oc, gc, L):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    for step in range(2):
        q = S.gen_q(wl, 0, 0, step=step)
        ref = oc.qk(q, SCALE)
        scores = torch.full((wl.n_q_heads, L + 3), -7.0, device="cuda")
        K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
        got = scores.cpu().numpy()
        assert np.all(got[:, L:] == -7.0)
        ok, worst = matvec_close(got[:, :L], ref)
        assert ok, f"qk worst error / bound = {worst:.3f}"
        p = O.softmax(ref)
        out = torch.empty((wl.n_q_heads, 128), device="cuda")
        K.kvq_pv_matvec(gc, torch.from_numpy(p).cuda(), out)
        ok, worst = matvec_close(out.cpu().numpy(), oc.pv(p))
        assert ok, f"pv worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("bits,L", [(3, 333), (4, 200)])
def test_empty_and_full_tokens(bits, L):
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4, bits=bits)
    st = Setup(wl)
    rng = np.random.default_rng(7)
    k, empty, full = _crafted_keys(st, L, rng)
    v = st.v(0, L)
    cap = 512
    oc, gc = _run(st, k, v, L, cap)
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    cnt = np.diff(oc.k_ptr[:L + 1].astype(np.int64))
    assert np.all(cnt[empty] == 0) and np.all(cnt[:3] == 0) and np.all(cnt[L - 2:] == 0)   # the plant took
    assert np.all(cnt[full] == wl.D)
    _check_matvecs(st, oc, gc, L)


def test_many_outliers_per_token_need_several_batches():
    # 8 % outliers on D = 1024: 82 entries per token, so eight tokens exceed one batch of either kernel
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8, outlier_fraction=0.08)
    st = Setup(wl)
    L = 700
    oc, gc = _run(st, st.k(0, L), st.v(0, L), L, 768)
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    cnt_k = np.diff(oc.k_ptr[:L + 1].astype(np.int64))
    cnt_v = np.diff(oc.v_ptr[:L + 1].astype(np.int64))
    assert cnt_k.mean() > 60 and np.all(cnt_v == 2 * st.k_side) and 2 * st.k_side > 64
    _check_matvecs(st, oc, gc, L)


def test_sparse_arrays_without_slack():
    """The sparse arrays end exactly at the last entry: batched loads near the end must stay inside."""
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    L = 391
    k, v = st.k(0, L), st.v(0, L)
    # first pass through the oracle alone tells how many entries there will be
    probe = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, 512, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                          st.s, st.z, st.lo, st.hi)
    probe.append_k(k); probe.append_v(v)
    nnz_k, nnz_v = int(probe.k_ptr[L]), int(probe.v_ptr[L])
    oc, gc = _run(st, k, v, L, 512, cap_nnz_k=nnz_k, cap_nnz_v=nnz_v)
    assert gc.status() == 0                     # exactly full is not an overflow
    assert not compare_caches(oc, gc)
    _check_matvecs(st, oc, gc, L)


def test_gqa_with_crafted_tokens():
    wl = S.workload("c4", n_kv_heads=2, n_q_heads=8)
    st = Setup(wl)
    L = 150
    rng = np.random.default_rng(11)
    k, empty, full = _crafted_keys(st, L, rng)
    oc, gc = _run(st, k, st.v(0, L), L, 256)
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    _check_matvecs(st, oc, gc, L)


def test_storage_past_the_last_token_is_never_used():
    """Odd token count: the last token shares its code words and its (scale, zero-point) pair slot
    with a token that does not exist yet.  Whatever the buffers hold there (NaN scale, set bits in the
    codes) must not reach the result of either mat-vec or of the fused call."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    L = 333
    oc, gc = _run(st, st.k(0, L), st.v(0, L), L, 512)
    assert not compare_caches(oc, gc)
    gc.v_sz.view(torch.int16)[2 * L:] = 0x7E00                    # fp16 NaN in every later (scale, zero-point)
    q = S.gen_q(wl, 0, 0)
    ref_scores = oc.qk(q, SCALE)
    p = O.softmax(ref_scores)
    out = torch.empty((wl.n_q_heads, 128), device="cuda")
    K.kvq_pv_matvec(gc, torch.from_numpy(p).cuda(), out)
    ok, worst = matvec_close(out.cpu().numpy(), oc.pv(p))
    assert ok, f"pv worst error / bound = {worst:.3f}"
    scores = torch.zeros((wl.n_q_heads, L), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), SCALE, scores, out)
    ok, worst = matvec_close(out.cpu().numpy(), oc.pv(p), rel=2e-3)
    assert ok, f"fused worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("L_full,extra", [(100, 4), (37, 0)])
def test_value_tokens_with_unequal_outlier_counts(L_full, extra):
    """The Value outlier array runs full part way through token L_full: the tokens before it keep their
    2 * k_side outliers, that token `extra` of them, the later ones none.  The sparse Value kernel
    takes an entry's token from a division where every token of a range has the same count and from
    the pointers otherwise: both kinds of range occur here, and a range that is even except for its
    last token.  The oracle does not model a full array; what the format prescribes for one (pointers
    clamped to the capacity, i.e. the excess dropped, highest channels first) is applied to the
    oracle's cache here."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    L, cap = 333, 512
    cap_nnz_v = 2 * st.k_side * L_full + extra
    k, v = st.k(0, L), st.v(0, L)
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi)
    oc.append_k(k); oc.append_v(v)
    oc.v_ptr = np.minimum(oc.v_ptr, cap_nnz_v).astype(oc.v_ptr.dtype)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, wl.D * cap, cap_nnz_v=cap_nnz_v)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    for t0, T in ((0, 64), (64, 130), (194, 1), (195, L - 195)):
        K.kvq_quantize_append_k(gc, torch.from_numpy(k[t0:t0 + T]).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v[t0:t0 + T]).cuda())
    torch.cuda.synchronize()
    assert gc.status() == 4                                    # KVQ_ERR_NNZ_OVERFLOW: reported, the excess dropped
    assert np.array_equal(gc.v_ptr.cpu().numpy()[:L + 1].astype(np.int64), oc.v_ptr[:L + 1].astype(np.int64))
    idx, val = gc.sparse_entries("v", cap_nnz_v)
    assert np.array_equal(idx.cpu().numpy().view(np.uint16), oc.v_idx[:cap_nnz_v])
    assert np.array_equal(val.cpu().numpy().view(np.uint16), oc.v_val[:cap_nnz_v])
    cnt = np.diff(oc.v_ptr[:L + 1].astype(np.int64))
    assert np.all(cnt[:L_full] == 2 * st.k_side) and cnt[L_full] == extra and np.all(cnt[L_full + 1:] == 0)
    _check_matvecs(st, oc, gc, L)
    q = S.gen_q(wl, 0, 0)
    scores = torch.zeros((wl.n_q_heads, L), device="cuda")
    out = torch.empty((wl.n_q_heads, 128), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), SCALE, scores, out)
    ok, worst = matvec_close(out.cpu().numpy(), oc.pv(O.softmax(oc.qk(q, SCALE))), rel=2e-3)
    assert ok, f"fused worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("heads,L", [((4, 4), 333), ((2, 8), 150)])
def test_long_sub_ranges_with_empty_and_full_tokens(heads, L):
    """Key outlier arrays sized for fewer than 16 outliers per token make the sparse Key kernel walk
    sub-ranges of 32 tokens, where an entry's token comes from a scatter of the token pointers and a
    prefix maximum over the lanes.  Planted: runs of tokens without any outlier (equal pointers), at
    the very start and end too, and tokens whose every channel is an outlier (several groups of 64
    entries inside one token)."""
    wl = S.workload("c2", n_kv_heads=heads[0], n_q_heads=heads[1])
    st = Setup(wl)
    rng = np.random.default_rng(23)
    k, empty, full = _crafted_keys(st, L, rng)
    v = st.v(0, L)
    cap = 512
    probe = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                          st.s, st.z, st.lo, st.hi)
    probe.append_k(k)
    nnz_k = int(probe.k_ptr[L])
    assert nnz_k // cap < 16                                    # the 32-token sub-ranges are taken
    oc, gc = _run(st, k, v, L, cap, cap_nnz_k=nnz_k)
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    cnt = np.diff(oc.k_ptr[:L + 1].astype(np.int64))
    assert np.all(cnt[np.setdiff1d(empty, full)] == 0) and np.all(cnt[:3] == 0) and np.all(cnt[L - 2:] == 0)
    assert np.all(cnt[full] == wl.D)
    _check_matvecs(st, oc, gc, L)
