"""The per-kernel timing aid: one event pair per call out of a ring, read back after the calls."""
import numpy as np
import pytest

import kvq_synth as S
from kvq_testlib import Setup

pytestmark = pytest.mark.gpu


def test_profile_ring_records_every_call_and_wraps():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    gc = st.gpu_cache(512)
    K.kvq_quantize_append_kv(gc, torch.from_numpy(st.k(0, 300)).cuda(), torch.from_numpy(st.v(0, 300)).cuda())
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores = torch.zeros((4, 512), device="cuda")
    out = torch.zeros((4, 128), device="cuda")
    ref = None
    K.kvq_profile_enable(True)
    try:
        assert K.kvq_profile_read_all_us(0) == [] and K.kvq_profile_read_all_us(1) == []
        with pytest.raises(K.KvqError):
            K.kvq_profile_last_ms(0)                              # nothing recorded yet
        for i in range(5):
            K.kvq_attention_decode(gc, q, 0.1, scores, out)
        ref = out.clone()
        qk, pv = K.kvq_profile_read_all_us(0), K.kvq_profile_read_all_us(1)
        assert len(qk) == 5 and len(pv) == 5
        assert all(0.5 < t < 5000.0 for t in qk + pv)             # microseconds of a tiny kernel
        assert K.kvq_profile_last_ms(0) * 1e3 == pytest.approx(qk[-1])
        for i in range(300):                                      # more calls than the ring holds
            K.kvq_qk_matvec(gc, q, 0.1, scores)
        qk = K.kvq_profile_read_all_us(0)
        assert len(qk) == 256 and len(K.kvq_profile_read_all_us(1)) == 5
        lib, ms = K.load_library(), __import__("ctypes").c_float()
        assert lib.kvq_profile_read_ms(0, 10, __import__("ctypes").byref(ms)) == 1     # overwritten: INVALID_ARG
        assert lib.kvq_profile_read_ms(0, 305, __import__("ctypes").byref(ms)) == 1    # not recorded yet
        assert lib.kvq_profile_read_ms(2, 0, __import__("ctypes").byref(ms)) == 1
    finally:
        K.kvq_profile_enable(False)
    K.kvq_attention_decode(gc, q, 0.1, scores, out)               # results do not depend on the bracket
    assert torch.equal(out, ref)
    K.kvq_profile_enable(True)                                    # enabling again starts from zero
    assert K.kvq_profile_read_all_us(0) == []
    K.kvq_profile_enable(False)


def test_kernel_spans_agree_with_the_event_intervals():
    """The dense kernels' own spans (first wavefront start to last wavefront end on the GPU wall clock)
    against the HIP-event interval around the same launches: the span is never longer than the interval
    (which also holds the launch latency) and not much shorter on a kernel of some tens of microseconds."""
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=8, n_q_heads=8)
    st = Setup(wl)
    L = 16384
    gc = st.gpu_cache(L + 128)
    for t0 in range(0, L, 4096):
        K.kvq_quantize_append_kv(gc, torch.from_numpy(st.k(t0, 4096)).cuda(), torch.from_numpy(st.v(t0, 4096)).cuda())
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores = torch.zeros((8, L + 128), device="cuda")
    out = torch.zeros((8, 128), device="cuda")
    for _ in range(3):
        K.kvq_attention_decode(gc, q, 0.1, scores, out)
    ref = out.clone()
    K.kvq_profile_enable(True, spans=True)
    try:
        for _ in range(20):
            K.kvq_attention_decode(gc, q, 0.1, scores, out)
        torch.cuda.synchronize()
        for which in (0, 1):
            spans, evs = K.kvq_profile_read_all_spans_us(which), K.kvq_profile_read_all_us(which)
            assert len(spans) == 20 and len(evs) == 20
            # sanity bounds only: the two figures come from different clocks and a slow launch on a
            # busy machine must not fail a correctness run
            assert all(0.5 < s < 20000.0 for s in spans)
            assert all(0.5 < e < 200000.0 for e in evs)
    finally:
        K.kvq_profile_enable(False)
    assert torch.equal(out, ref)
    K.kvq_profile_enable(True, spans=True, events=False)          # spans only: no event intervals to read
    try:
        K.kvq_attention_decode(gc, q, 0.1, scores, out)
        assert len(K.kvq_profile_read_all_spans_us(0)) == 1
        with pytest.raises(K.KvqError):
            K.kvq_profile_read_all_us(0)
    finally:
        K.kvq_profile_enable(False)
