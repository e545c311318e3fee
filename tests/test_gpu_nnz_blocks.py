"""Blocked outlier storage (paper App. "Limitations": the sparse matrix allocated in blocks, so that an
append copies nothing already stored): entry e lives in block e >> shift, found through a table of block
addresses.  A cache that starts with one block per array and gets more between appends holds, bit for bit,
what the oracle's flat arrays hold; the mat-vecs give, bit for bit, what they give on flat arrays (the
accumulation is order-free fixed point) and agree with the oracle; no block ever moves."""
import ctypes as C

import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)
BE = 1024                       # entries per block: the smallest the library takes


def _caches(st, cap, be=BE, n_sink=0):
    """(oracle cache, blocked GPU cache with ONE block per array)."""
    import paper_2401_18079_amd as K
    wl = st.wl
    full_k, full_v = wl.D * cap, max(8, 2 * st.k_side * cap)
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=full_k, cap_nnz_v=full_v, n_sink=n_sink)
    bc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, cap_nnz_k=1, cap_nnz_v=1,
                    n_sink=n_sink, nnz_block_entries=be, nnz_table_slots=max(8, (full_k + be - 1) // be + 2))
    K.kvq_lut_load(bc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    assert bc.c.cap_nnz_k == be and bc.c.cap_nnz_v == be and bc.c.nnz_block_shift == be.bit_length() - 1
    return oc, bc


def _flat_twin(st, bc, k, v, chunks):
    """A flat cache of the blocked cache's final capacities (the launch plans look at the capacity, and
    bit-for-bit equality of the mat-vecs needs the same plan), filled with the same appends."""
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    fc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, bc.c.cap_tokens, st.k_side, wl.rope_base, bc.c.cap_nnz_k,
                    cap_nnz_v=bc.c.cap_nnz_v, n_sink=bc.c.n_sink)
    K.kvq_lut_load(fc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    t0, i = 0, 0
    while t0 < k.shape[0]:
        T = min(chunks[i % len(chunks)], k.shape[0] - t0)
        K.kvq_quantize_append_kv(fc, torch.from_numpy(k[t0:t0 + T]).cuda(), torch.from_numpy(v[t0:t0 + T]).cuda())
        t0 += T
        i += 1
    assert fc.status() == 0
    return fc


def _append_all(st, oc, bc, k, v, chunks):
    """Append in the given chunk sizes (cycled); odd chunks through the combined call.  The blocked cache
    gets room for each chunk's worst case just before it."""
    import torch
    import paper_2401_18079_amd as K
    L, D, t0, i, grown = k.shape[0], st.wl.D, 0, 0, 0
    first = {n: bc.blocks[n][0].data_ptr() for n in bc.blocks}
    while t0 < L:
        T = min(chunks[i % len(chunks)], L - t0)
        kk, vv = k[t0:t0 + T], v[t0:t0 + T]
        oc.append_k(kk); oc.append_v(vv)
        grown += bc.ensure_nnz_room(T * D, T * 2 * st.k_side)
        kd, vd = torch.from_numpy(kk).cuda(), torch.from_numpy(vv).cuda()
        if i % 2:
            K.kvq_quantize_append_kv(bc, kd, vd)
        else:
            K.kvq_quantize_append_k(bc, kd)
            K.kvq_quantize_append_v(bc, vd)
        t0 += T
        i += 1
    torch.cuda.synchronize()
    assert all(bc.blocks[n][0].data_ptr() == p for n, p in first.items())      # the first block never moved
    return grown


def _matvecs_agree(st, oc, fc, bc, L, cap):
    import torch
    import paper_2401_18079_amd as K
    wl = st.wl
    for step in range(2):
        q = S.gen_q(wl, 0, 0, step=step)
        qd = torch.from_numpy(q).cuda()
        ref = oc.qk(q, SCALE)
        got = {}
        for name, c in (("flat", fc), ("blocked", bc)):
            scores = torch.full((wl.n_q_heads, cap), -7.0, device="cuda")
            K.kvq_qk_matvec(c, qd, SCALE, scores)
            out = torch.empty((wl.n_q_heads, 128), device="cuda")
            K.kvq_pv_matvec(c, torch.from_numpy(O.softmax(ref)).cuda(), out)
            fs = torch.zeros((wl.n_q_heads, cap), device="cuda")
            fo = torch.zeros((wl.n_q_heads, 128), device="cuda")
            K.kvq_attention_decode(c, qd, SCALE, fs, fo)
            no = torch.zeros((wl.n_q_heads, 128), device="cuda")
            K.kvq_attention_decode_noalloc(c, qd, SCALE, torch.zeros_like(fs), no)
            got[name] = (scores, out, fs, fo, no)
        for a, b in zip(got["flat"], got["blocked"]):
            assert torch.equal(a, b)                                  # same entries, order-free sums
        scores, out, _, fo, _ = got["blocked"]
        ok, worst = matvec_close(scores.cpu().numpy()[:, :L], ref)
        assert ok, f"qk worst error / bound = {worst:.3f}"
        ok, worst = matvec_close(out.cpu().numpy(), oc.pv(O.softmax(ref)))
        assert ok, f"pv worst error / bound = {worst:.3f}"
        ok, worst = matvec_close(fo.cpu().numpy(), oc.pv(O.softmax(ref)), rel=2e-3)
        assert ok, f"fused outputs: worst error / bound = {worst:.3f}"


@pytest.mark.parametrize("bits,heads,frac,L,chunks", [
    (3, 4, 0.0625, 1536, (1, 1, 3, 64, 1, 200, 1, 130)),     # D = 512; Value entries fill 48 blocks exactly
    (2, 8, 0.03, 1300, (1, 2, 1100, 1, 70)),                 # D = 1024; one call of >= 1024 tokens (wavefront-per-token Keys)
    (4, 16, 0.01, 420, (1, 1, 2, 1, 37, 1, 260, 5)),         # D = 2048; the wide single-token workgroups
])
def test_blocked_cache_holds_what_flat_arrays_hold(bits, heads, frac, L, chunks):
    wl = S.workload("c2", n_kv_heads=heads, n_q_heads=heads, bits=bits, outlier_fraction=frac)
    st = Setup(wl)
    cap = (L + 127) // 128 * 128
    oc, bc = _caches(st, cap)
    grown = _append_all(st, oc, bc, st.k(0, L), st.v(0, L), chunks)
    assert grown >= 2 and len(bc.blocks["k_idx"]) >= 5 and len(bc.blocks["v_val"]) >= 5      # grew, several times
    assert bc.status() == 0
    fc = _flat_twin(st, bc, st.k(0, L), st.v(0, L), chunks)
    assert not compare_caches(oc, bc)
    nk, nv = int(oc.k_ptr[L]), int(oc.v_ptr[L])
    assert nk > 4 * BE and nv > 4 * BE                       # entries really span several blocks
    # tokens whose Key entries straddle a block boundary exist (Value entries: a fixed count per token,
    # which may divide the block size)
    p = oc.k_ptr[:L + 1].astype(np.int64)
    assert np.any(((p[:-1] // BE) != ((p[1:] - 1) // BE)) & (p[1:] > p[:-1]))
    _matvecs_agree(st, oc, fc, bc, L, cap)


def test_last_block_exactly_full():
    """Entries end exactly at the end of the last block on both sides: the batched loads of the two sparse
    kernels near the end stay inside it."""
    import torch
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=8, outlier_fraction=0.0625)       # 32 Value entries a token
    st = Setup(wl)
    L, cap = 160, 256
    k = np.tile(np.asarray(st.z, dtype=np.float16), (L, 1))                         # mid-points: no Key outliers ...
    hi, lo = (np.asarray(a, dtype=np.float16).astype(np.float32) for a in (st.hi, st.lo))
    for t in (5, 6, 77, 159):                                                       # ... but four rows full of them
        k[t] = (hi + 4.0 * (hi - lo) + 1.0).astype(np.float16)
    oc, bc = _caches(st, cap)
    import paper_2401_18079_amd as K
    t0, v = 0, st.v(0, L)
    for T in (7, 1, 64, 88):
        kk, vv = k[t0:t0 + T], v[t0:t0 + T]
        oc.append_k(kk); oc.append_v(vv)
        # room for exactly what this chunk stores (known here from the oracle), so nothing is left over
        bc.ensure_nnz_room(int(oc.k_ptr[t0 + T]) - int(oc.k_ptr[t0]), int(oc.v_ptr[t0 + T]) - int(oc.v_ptr[t0]))
        K.kvq_quantize_append_kv(bc, torch.from_numpy(kk).cuda(), torch.from_numpy(vv).cuda())
        t0 += T
    fc = _flat_twin(st, bc, k, v, (7, 1, 64, 88))
    assert int(oc.k_ptr[L]) == 4 * wl.D == 2 * BE == bc.c.cap_nnz_k
    assert int(oc.v_ptr[L]) == 32 * L == 5 * BE == bc.c.cap_nnz_v
    assert bc.status() == 0 and not compare_caches(oc, bc)
    _matvecs_agree(st, oc, fc, bc, L, cap)


def test_blocked_cache_with_sink_tokens_and_gqa():
    wl = S.workload("c4", n_kv_heads=4, n_q_heads=16, outlier_fraction=0.04)
    st = Setup(wl)
    L, cap = 900, 1024
    oc, bc = _caches(st, cap, n_sink=3)
    _append_all(st, oc, bc, st.k(0, L), st.v(0, L), (1, 1, 1, 1, 300, 1))
    assert bc.status() == 0 and not compare_caches(oc, bc)
    fc = _flat_twin(st, bc, st.k(0, L), st.v(0, L), (1, 1, 1, 1, 300, 1))
    _matvecs_agree(st, oc, fc, bc, L, cap)


def test_overflow_of_the_last_block_is_reported():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4, outlier_fraction=0.0625)
    st = Setup(wl)
    _, bc = _caches(st, 256)
    K.kvq_quantize_append_v(bc, torch.from_numpy(st.v(0, 40)).cuda())              # 1280 entries, room for 1024
    assert bc.status() == 4 and bc.nnz_used()[1] == BE


def test_descriptor_checks():
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=4, n_q_heads=4)
    st = Setup(wl)
    _, bc = _caches(st, 256)
    lib = K.load_library()
    k = torch.from_numpy(st.k(0, 1)).cuda()

    def status_with(**fields):
        old = {n: getattr(bc.c, n) for n in fields}
        for n, v in fields.items():
            setattr(bc.c, n, v)
        try:
            return lib.kvq_quantize_append_k(C.byref(bc.c), k.data_ptr(), 1, None)
        finally:
            for n, v in old.items():
                setattr(bc.c, n, v)

    assert status_with(nnz_block_shift=9) == 1 and status_with(nnz_block_shift=31) == 1
    assert status_with(cap_nnz_k=BE + 8) == 1 and status_with(cap_nnz_v=0) == 1
    assert status_with(k_idx_blocks=None) == 1 and status_with(v_val_blocks=bc.tables["v_val"].data_ptr() + 4) == 1
    assert bc.n_tokens_k == 0
    assert status_with() == 0 and bc.n_tokens_k == 1                                # untouched descriptor works
