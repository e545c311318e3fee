"""GPU parity for the fused decode-attention call (scores, softmax and output in one call: the
generation-time attention of paper Sec. 3 with the two quantized mat-vecs of App. "Kernel
Implementation Details").

Two comparisons per case.  (1) Against the CPU oracle's chain qk -> softmax -> pv.  The oracle's
softmax sees the oracle's scores, the kernels' softmax sees the kernels' scores, which differ by up
to the mat-vec tolerance delta = 1e-3 (|s| + rms(s)); a score error delta multiplies a weight by
e^delta, so the chained output gets twice the mat-vec tolerance, 2e-3 (the same bound the smoke test
uses for the three separate calls).  (2) Against the three separate calls on the same GPU cache, which
start from bit-identical scores: only the order of the exponential sums differs, so 2e-5.
"""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)
CHAIN_TOL = 2e-3
SAME_SCORES_TOL = 2e-5


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


def _separate_calls(gc, q_dev, scale, L, ld):
    import torch
    import paper_2401_18079_amd as K
    Hq = gc.c.n_q_heads
    scores = torch.zeros((Hq, ld), device="cuda")
    probs = torch.zeros_like(scores)
    out = torch.zeros((Hq, 128), device="cuda")
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(Hq, ld), dtype=torch.uint8, device="cuda")
    K.kvq_qk_matvec(gc, q_dev, scale, scores)
    K.kvq_softmax_f32(scores, probs, L, ws)
    K.kvq_pv_matvec(gc, probs, out)
    return scores, out


def _check_fused(st, oc, gc, L, scale=SCALE, q_gain=1.0, steps=2):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    assert gc.status() == 0
    assert not compare_caches(oc, gc)
    ld = L + 5
    for step in range(steps):
        q = (S.gen_q(wl, 0, 0, step=step) * q_gain).astype(np.float32)
        q_dev = torch.from_numpy(q).cuda()
        scores = torch.full((wl.n_q_heads, ld), -3.0, device="cuda")
        out = torch.full((wl.n_q_heads, 128), 77.0, device="cuda")
        K.kvq_attention_decode(gc, q_dev, scale, scores, out)
        got = out.cpu().numpy()
        # the oracle's chain
        ref_scores = oc.qk(q, scale)
        ref = oc.pv(O.softmax(ref_scores))
        ok, worst = matvec_close(got, ref, rel=CHAIN_TOL)
        assert ok, f"fused output against the oracle chain: worst error / bound = {worst:.3f}"
        # the three separate calls: same scores bit for bit, same output up to summation order
        s3, o3 = _separate_calls(gc, q_dev, scale, L, ld)
        assert torch.equal(scores[:, :L], s3[:, :L])
        assert torch.all(scores[:, L:] == -3.0)                  # nothing written past the tokens
        ok, worst = matvec_close(got, o3.cpu().numpy(), rel=SAME_SCORES_TOL)
        assert ok, f"fused output against the separate calls: worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("name,ov,n_sink,L,chunks", [
    ("c2", dict(n_kv_heads=8, n_q_heads=8), 0, 2500, [1, 700, 64]),            # three 1024-token tiles, ragged tail
    ("c2", dict(n_kv_heads=4, n_q_heads=4, bits=2), 0, 1100, [300]),
    ("c3", dict(n_kv_heads=8, n_q_heads=8, outlier_fraction=0.004), 0, 777, [777]),    # 4-bit, 8 heads per workgroup
    ("c4", dict(n_kv_heads=2, n_q_heads=8), 0, 1300, [2, 640]),                # grouped-query attention
    ("c2", dict(n_kv_heads=2, n_q_heads=16), 0, 300, [150]),                    # eight query heads per KV head
    ("c2", dict(n_kv_heads=4, n_q_heads=8), 0, 450, [450]),                     # two per KV head (3-bit)
    ("c3", dict(n_kv_heads=2, n_q_heads=8, outlier_fraction=0.004), 0, 390, [390]),   # four per KV head, 4-bit
    ("c2", dict(n_kv_heads=2, n_q_heads=8, bits=2), 2, 333, [333]),             # four per KV head, 2-bit, sinks
    ("c2", dict(n_kv_heads=3, n_q_heads=3), 0, 700, [350]),                     # head count that fits no group: one head per workgroup
    ("c2", dict(n_kv_heads=4, n_q_heads=4, outlier_fraction=0.0), 0, 129, [5]), # no outliers: the sparse Key kernel is skipped
    ("c2", dict(n_kv_heads=8, n_q_heads=8), 1, 1500, [1, 2, 500]),              # one attention-sink token
    ("c4", dict(n_kv_heads=2, n_q_heads=8), 4, 200, [2, 64]),
    ("c2", dict(n_kv_heads=4, n_q_heads=4), 4, 3, [1]),                         # fewer tokens than sinks: every token in fp16
    ("c2", dict(n_kv_heads=4, n_q_heads=4), 0, 1, [1]),                         # a single token: its weight is exactly 1
])
def test_fused_decode_matches_oracle_chain(name, ov, n_sink, L, chunks):
    wl = S.workload(name, **ov)
    st = Setup(wl)
    cap = (L + 127) // 128 * 128 + 128
    oc, gc = _pair(st, cap, n_sink, L, chunks)
    _check_fused(st, oc, gc, L)


@pytest.mark.parametrize("n_sink", [0, 3])
def test_fused_decode_with_more_than_64_maxima_per_head(n_sink):
    """Four heads in one head group and 69 tiles of 1024 tokens: the dense Key kernel runs 69 workgroups
    per head, so every consumer merges more score maxima than a wavefront has lanes."""
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    L = 69 * 1024 + 77
    oc, gc = _pair(st, 70 * 1024, n_sink, L, [4096])
    _check_fused(st, oc, gc, L, steps=1)


@pytest.mark.parametrize("name,L", [("c2", 6000), ("c3", 10500)])
def test_mid_context_uses_the_half_size_head_groups(name, L):
    """Full-width layers (32 heads) at contexts of a few thousand tokens: too short for the widest
    head grouping of the dense Key kernel, long enough for the one with half as many heads per
    workgroup and tiles of 512 tokens (3-bit from 5K tokens, 4-bit from 10K)."""
    wl = S.workload(name)
    st = Setup(wl)
    cap = (L + 127) // 128 * 128 + 128
    oc, gc = _pair(st, cap, 0, L, [4096])
    _check_fused(st, oc, gc, L, steps=1)


@pytest.mark.parametrize("n_sink", [0, 2])
def test_fused_decode_with_large_scores(n_sink):
    """Scores of magnitude in the hundreds: exp overflows fp32 unless the maximum is subtracted, and
    nearly all weight sits on a handful of tokens."""
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    L = 1300
    oc, gc = _pair(st, 1536, n_sink, L, [650])
    q = S.gen_q(wl, 0, 0) * 40.0
    peak = np.abs(oc.qk(q.astype(np.float32), SCALE)).max()
    assert peak > 100.0, peak                      # the case is what it claims to be
    _check_fused(st, oc, gc, L, q_gain=40.0, steps=1)


def test_fused_decode_empty_cache_and_argument_errors():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    gc = st.gpu_cache(256)
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores = torch.full((4, 256), 9.0, device="cuda")
    out = torch.full((4, 128), 9.0, device="cuda")
    K.kvq_attention_decode(gc, q, SCALE, scores, out)           # empty cache: zeros, scores untouched
    assert torch.all(out == 0.0) and torch.all(scores == 9.0)
    K.kvq_quantize_append_k(gc, torch.from_numpy(st.k(0, 3)).cuda())
    with pytest.raises(K.KvqError):                             # 3 Keys, 0 Values
        K.kvq_attention_decode(gc, q, SCALE, scores, out)
    K.kvq_quantize_append_v(gc, torch.from_numpy(st.v(0, 3)).cuda())
    K.kvq_attention_decode(gc, q, SCALE, scores, out)
    with pytest.raises(K.KvqError):                             # leading dimension below the token count
        K.kvq_attention_decode(gc, q, SCALE, torch.zeros((4, 2), device="cuda"), out)
    ws_bytes = gc.c.workspace_bytes
    gc.c.workspace_bytes = 1024                                 # workspace too small for the statistics
    with pytest.raises(K.KvqError):
        K.kvq_attention_decode(gc, q, SCALE, scores, out)
    gc.c.workspace_bytes = ws_bytes


def test_fused_decode_is_deterministic():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    L = 2100
    _, gc = _pair(st, 2304, 1, L, [700])
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    outs = []
    for _ in range(3):
        scores = torch.zeros((8, L), device="cuda")
        out = torch.zeros((8, 128), device="cuda")
        K.kvq_attention_decode(gc, q, SCALE, scores, out)
        outs.append(out.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
