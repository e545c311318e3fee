"""kvq_attention_decode_noalloc (the entry point for callers that cannot allocate: its scratch is a
static array inside the library) against kvq_attention_decode, through the C ABI: same kernels, so the
outputs and the scores must be identical bit for bit, on two calls in a row, the second on a smaller
input, and with the descriptor's workspace pointer taken away."""
import numpy as np
import pytest

import kvq_synth as S
from kvq_testlib import Setup, fill_both

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


def _both(st, gc, L, cap, step):
    import torch
    import paper_2401_18079_amd as K
    Hq = st.wl.n_q_heads
    q = torch.from_numpy(S.gen_q(st.wl, 0, 0, step=step)).cuda()
    s_ref = torch.full((Hq, cap), 7.0, device="cuda"); s_new = torch.full((Hq, cap), 7.0, device="cuda")
    o_ref = torch.zeros((Hq, 128), device="cuda"); o_new = torch.full((Hq, 128), -1.0, device="cuda")
    K.kvq_attention_decode(gc, q, SCALE, s_ref, o_ref)
    torch.cuda.synchronize()
    ws, wsb = gc.c.workspace, gc.c.workspace_bytes
    gc.c.workspace, gc.c.workspace_bytes = None, 0           # the new entry point must not need it
    try:
        K.kvq_attention_decode_noalloc(gc, q, SCALE, s_new, o_new)
        torch.cuda.synchronize()
    finally:
        gc.c.workspace, gc.c.workspace_bytes = ws, wsb
    assert torch.equal(s_new, s_ref)
    assert torch.equal(o_new, o_ref)
    assert torch.isfinite(o_new).all() and float(o_new.abs().max()) > 0


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    import torch
    import paper_2401_18079_amd as K
    # first call: 32 query heads (the limit), a context that spans many slabs and a ragged tail
    wl = S.workload("c2", n_kv_heads=32, n_q_heads=32)
    st = Setup(wl)
    L1, cap1 = 5000, 5120
    g1 = st.gpu_cache(cap1)
    fill_both(st, None, g1, L1, [4096])
    _both(st, g1, L1, cap1, 0)
    # second call right after it, on a smaller input (fewer heads, fewer tokens, another code width):
    # whatever the first call left in the static array must not show
    wl2 = S.workload("c4", n_kv_heads=2, n_q_heads=8)
    st2 = Setup(wl2)
    L2, cap2 = 333, 384
    g2 = st2.gpu_cache(cap2)
    fill_both(st2, None, g2, L2, [333])
    _both(st2, g2, L2, cap2, 1)
    # and the first input again
    _both(st, g1, L1, cap1, 2)
    # beyond the stated limit: a clear error, nothing launched
    wl3 = S.workload("c2", n_kv_heads=64, n_q_heads=64)
    st3 = Setup(wl3)
    g3 = st3.gpu_cache(128)
    q = torch.zeros((64, 128), device="cuda"); sc = torch.zeros((64, 128), device="cuda"); o = torch.zeros((64, 128), device="cuda")
    with pytest.raises(K.KvqError) as e:
        K.kvq_attention_decode_noalloc(g3, q, SCALE, sc, o)
    assert "capacity" in str(e.value)
