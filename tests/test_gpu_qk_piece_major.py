"""GPU parity for the piece-major dense Key kernel (3-bit codes, tiles of 1024 tokens, a lane's
(cos, sin) advanced from tile to tile by a rotation instead of being recomputed), in the launch
configurations that select it: contexts of 20+ tiles with the bench workload's head shape.  Every score
against the oracle at contexts where a workgroup's block holds one tile, two or three tiles (ragged
blocks), and sampled windows where workgroups run more than one block; grouped-query shapes; the fused
call's statistics; attention-sink tokens."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, matvec_close
from test_gpu_fullsize import _sampled_full_size_parity, WIN

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


def _every_score(wl, L, n_sink=0):
    import torch
    import paper_2401_18079_amd as K
    st = Setup(wl)
    cap = ((L + 127) // 128) * 128
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=st.cap_nnz_k(cap), n_sink=n_sink)
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap), n_sink=n_sink)
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0 = 0
    while t0 < L:
        T = min(4096, L - t0)
        k, v = st.k(t0, T), st.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        t0 += T
    torch.cuda.synchronize()
    assert gc.status() == 0
    q = S.gen_q(wl, 0, 0)
    ref = oc.qk(q, SCALE)
    scores = torch.full((wl.n_q_heads, cap + 3), 5.0, device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
    got = scores.cpu().numpy()
    assert np.all(got[:, L:] == 5.0)
    ok, worst = matvec_close(got[:, :L], ref)
    assert ok, f"scores: worst error / bound = {worst:.3f}"
    # the fused call (statistics variant of the kernel) against the oracle's chain
    ref_out = oc.pv(O.softmax(ref))
    out = torch.zeros((wl.n_q_heads, 128), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), SCALE, scores, out)
    ok, worst_f = matvec_close(out.cpu().numpy(), ref_out, rel=2e-3)
    assert ok, f"fused call: worst error / bound = {worst_f:.3f}"
    assert np.array_equal(scores.cpu().numpy()[:, :L], got[:, :L])          # same scores from both variants
    # the timing aid: this kernel's spans (earliest workgroup start to latest end, stamped through a
    # pointer the kernel reads from device memory); sanity bounds only, and results do not change
    K.kvq_profile_enable(True, spans=True)
    try:
        for _ in range(3):
            K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), SCALE, scores, out)
        K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
        spans, evs = K.kvq_profile_read_all_spans_us(0), K.kvq_profile_read_all_us(0)
        assert len(spans) == 4 and len(evs) == 4
        assert all(0.5 < x < 20000.0 for x in spans) and all(0.5 < x < 200000.0 for x in evs)
    finally:
        K.kvq_profile_enable(False)
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)          # the pointer is null again
    assert np.array_equal(scores.cpu().numpy()[:, :L], got[:, :L])
    return worst


def test_one_tile_per_block_and_a_ragged_last_tile():
    # 21 tiles: 21 workgroups per head group, one tile each; the last tile holds 533 tokens
    _every_score(S.workload("c2"), 20 * 1024 + 533)


def test_two_and_three_tiles_per_block_with_sink_tokens():
    # 45 tiles over 32 workgroups per head group: blocks of one and two tiles; two sink tokens
    _every_score(S.workload("c2"), 44 * 1024 + 1, n_sink=2)


def test_grouped_query_heads_share_the_fields():
    # 16 query heads on 8 KV heads (two KV heads x two query heads per workgroup), 3-bit
    _every_score(S.workload("c2", n_kv_heads=8, n_q_heads=16), 83 * 1024 + 77)


def test_several_blocks_per_workgroup_sampled():
    # 165 tiles over 32 workgroups: five or six tiles each = a full block and a ragged one
    wl = S.workload("c2")
    Lc = 164 * 1024 + 901
    starts = [0, (Lc // WIN) * WIN, 4096 - WIN, 4096, 5 * 1024, 5 * 1024 + 4096 - WIN, 10 * 1024 - WIN]
    _sampled_full_size_parity(wl, Lc, starts, n_random=6)
