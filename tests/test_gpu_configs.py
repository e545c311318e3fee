"""GPU parity on scaled-down versions of the remaining benchmark configurations."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, fill_both, compare_caches, matvec_close

pytestmark = pytest.mark.gpu
SCALE = 1.0 / np.sqrt(128.0)


def _attend(st, oc, gc, q, cap):
    import torch
    import paper_2401_18079_amd as K
    Hq, L = st.wl.n_q_heads, gc.n_tokens_k
    scores = torch.zeros((Hq, cap), device="cuda")
    probs = torch.zeros_like(scores)
    out = torch.zeros((Hq, 128), device="cuda")
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(Hq, cap), dtype=torch.uint8, device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
    K.kvq_softmax_f32(scores, probs, L, ws)
    K.kvq_pv_matvec(gc, probs, out)
    rs = oc.qk(q, SCALE)
    ro = oc.pv(O.softmax(rs))
    ok1, w1 = matvec_close(scores.cpu().numpy()[:, :L], rs)
    ok2, w2 = matvec_close(out.cpu().numpy(), ro, rel=2e-3)     # probabilities come from the GPU scores
    assert ok1 and ok2, (w1, w2)


def test_config3_shape_4bit_sparse_outliers_append_64_then_attend():
    """4-bit codes (split tables), 0.1 % outliers, online append of 64 tokens before the mat-vecs."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c3", context=3000)
    st = Setup(wl)
    cap = 3200
    oc, gc = st.oracle_cache(cap), st.gpu_cache(cap)
    fill_both(st, oc, gc, 3000 - 64, [1024])
    k, v = st.k(3000 - 64, 64), st.v(3000 - 64, 64)
    oc.append_k(k); oc.append_v(v)
    K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
    K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
    assert not compare_caches(oc, gc)
    _attend(st, oc, gc, S.gen_q(wl, 0, 0), cap)


def test_config4_shape_gqa_batch_of_sequences_2bit_rope_500000():
    """32 query heads over 8 KV heads, 2-bit codes, a batch of independent sequences (one cache each)."""
    wl = S.workload("c4", context=1500)
    st = Setup(wl)
    cap = 1536
    for seq in range(3):
        oc, gc = st.oracle_cache(cap), st.gpu_cache(cap)
        fill_both(st, oc, gc, 1500 - seq * 131, [512], seq=seq)
        assert not compare_caches(oc, gc)
        _attend(st, oc, gc, S.gen_q(wl, 0, seq), cap)


def test_config5_shape_layers_with_distinct_tables_decode_loop():
    """Several layers, each with its own look-up tables and channel constants: append one token, attend."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c5", context=700, n_kv_heads=8, n_q_heads=8)
    cap = 768
    layers = []
    for layer in range(3):
        st = Setup(wl, layer=layer)
        oc, gc = st.oracle_cache(cap), st.gpu_cache(cap)
        fill_both(st, oc, gc, 700, [700])
        layers.append((st, oc, gc))
    assert not np.array_equal(layers[0][0].lut_k, layers[1][0].lut_k)
    for step in range(2):
        for layer, (st, oc, gc) in enumerate(layers):
            n = 700 + step
            k, v = st.k(n, 1), st.v(n, 1)
            oc.append_k(k); oc.append_v(v)
            K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
            K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
            _attend(st, oc, gc, S.gen_q(wl, layer, 0, step=step), cap)
    for st, oc, gc in layers:
        assert not compare_caches(oc, gc)


def test_largest_append_batch_and_wide_models():
    """T = 4096 tokens in one call; 64 query heads; a single KV head with 8 query heads (GQA 8)."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=2, n_q_heads=2, context=4200)
    st = Setup(wl)
    oc, gc = st.oracle_cache(4224), st.gpu_cache(4224)
    fill_both(st, oc, gc, 4200, [4096, 104])
    assert not compare_caches(oc, gc)
    with pytest.raises(K.KvqError):
        K.kvq_quantize_append_k(gc, torch.zeros((4097, wl.D), dtype=torch.float16, device="cuda"))
    for ov in (dict(n_kv_heads=64, n_q_heads=64), dict(n_kv_heads=1, n_q_heads=8), dict(bits=4, n_kv_heads=3, n_q_heads=6),
               dict(bits=2, n_kv_heads=2, n_q_heads=16)):
        wl = S.workload("c2", context=333, **ov)
        st = Setup(wl)
        oc, gc = st.oracle_cache(384), st.gpu_cache(384)
        fill_both(st, oc, gc, 333, [200])
        assert not compare_caches(oc, gc), ov
        _attend(st, oc, gc, S.gen_q(wl, 0, 0), 384)


def test_results_are_reproducible_run_to_run():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8, context=5000)
    st = Setup(wl)
    gc = st.gpu_cache(5120)
    fill_both(st, None, gc, 5000, [2500])
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    a, b = torch.zeros((8, 5120), device="cuda"), torch.zeros((8, 5120), device="cuda")
    K.kvq_qk_matvec(gc, q, SCALE, a); K.kvq_qk_matvec(gc, q, SCALE, b)
    assert torch.equal(a, b)
    p = torch.softmax(a[:, :5000], dim=1).contiguous()
    oa, ob = torch.zeros((8, 128), device="cuda"), torch.zeros((8, 128), device="cuda")
    K.kvq_pv_matvec(gc, p, oa); K.kvq_pv_matvec(gc, p, ob)
    assert torch.equal(oa, ob)
