"""GPU parity with signpost tables that are NOT made of fp16 numbers: the tables a k-means solver
returns.  A cache stores its signposts as fp16 numbers (rounded once, when kvq_lut_load stores them;
the oracle does the same with its own conversion), so append, scores, outputs and the fused call all
see one table.  Cases: the library's own calibration output (kvq_calibrate_nuq) fed straight into
kvq_lut_load, and seeded fp32 draws; every code width; append bit-exact, mat-vecs at the 1e-3 tolerance."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import compare_caches, matvec_close

pytestmark = pytest.mark.gpu

SCALE = 1.0 / np.sqrt(128.0)


def _is_fp16(a):
    return np.array_equal(a, a.astype(np.float16).astype(np.float32))


def _calibrated_tables(bits):
    """Signposts from the library's own weighted k-means on synthetic calibration data, ends pinned to
    -1 / +1 the way a normalised vector touches its range (Keys and Values from different draws)."""
    import torch
    import paper_2401_18079_amd as K
    luts = []
    for which in (0, 1):
        x, w = S.gen_calibration(777 + 10 * bits + which, 1 << 18)
        c0 = np.linspace(-1, 1, 1 << bits).astype(np.float32)
        c = K.kvq_calibrate_nuq(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), bits, 8, c0)
        luts.append(np.asarray(c, dtype=np.float32))
    return luts


def _run_case(wl, lut_k, lut_v, L, chunks):
    import torch
    import paper_2401_18079_amd as K
    assert not _is_fp16(lut_k) and not _is_fp16(lut_v)
    lay = S.LayerInputs(wl)
    cap = ((L + 127) // 128) * 128
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, lay.k_side, wl.rope_base, lut_k, lut_v,
                       lay.s, lay.z, lay.lo, lay.hi, cap_nnz_k=lay.cap_nnz_k(cap))
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, lay.k_side, wl.rope_base, lay.cap_nnz_k(cap))
    K.kvq_lut_load(gc, lut_k, lut_v, lay.s, lay.z, lay.lo, lay.hi)
    t0, i = 0, 0
    while t0 < L:
        T = min(chunks[i % len(chunks)], L - t0)
        k, v = lay.k(t0, T), lay.v(t0, T)
        oc.append_k(k); oc.append_v(v)
        if i % 2:
            K.kvq_quantize_append_kv(gc, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
        else:
            K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
            K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        t0 += T
        i += 1
    torch.cuda.synchronize()
    assert gc.status() == 0
    bad = compare_caches(oc, gc)
    assert not bad, bad
    # the codes really depend on the rounding for some element, or the case proves nothing about it:
    # quantising with the table as handed over (the oracle's element-level function) must differ
    # somewhere in codes or residuals from the cache built on the stored table
    _, vc_raw, _, _, vv_raw = O.quantize_v(lay.v(0, min(L, 256)), wl.bits, lut_v, lay.k_side)
    vc_st = oc.unpack_v(0, min(L, 256))
    nv = int(oc.v_ptr[min(L, 256)])
    differs = (not np.array_equal(vc_raw, vc_st)) or (not np.array_equal(vv_raw, oc.v_val[:nv]))
    Hq = wl.n_q_heads
    q = S.gen_q(wl, 0, 0)
    ref_s = oc.qk(q, SCALE)
    scores = torch.zeros((Hq, cap), device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), SCALE, scores)
    ok, worst = matvec_close(scores.cpu().numpy()[:, :L], ref_s)
    assert ok, f"scores: worst error / bound = {worst:.3f}"
    ref_p = O.softmax(ref_s)
    ref_o = oc.pv(ref_p)
    pp = np.zeros((Hq, cap), dtype=np.float32); pp[:, :L] = ref_p
    out = torch.zeros((Hq, 128), device="cuda")
    K.kvq_pv_matvec(gc, torch.from_numpy(pp).cuda(), out)
    ok, worst_pv = matvec_close(out.cpu().numpy(), ref_o)
    assert ok, f"outputs: worst error / bound = {worst_pv:.3f}"
    fout = torch.zeros((Hq, 128), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), SCALE, scores, fout)
    ok, worst_f = matvec_close(fout.cpu().numpy(), ref_o, rel=2e-3)
    assert ok, f"fused call: worst error / bound = {worst_f:.3f}"
    print(f"bits {wl.bits}: scores {worst:.4f}, outputs {worst_pv:.4f}, fused {worst_f:.4f} of the bound")
    return differs


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_calibration_output_feeds_the_cache(bits):
    lut_k, lut_v = _calibrated_tables(bits)
    wl = S.workload("c2", bits=bits, n_kv_heads=8, n_q_heads=8)
    _run_case(wl, lut_k, lut_v, 700, [1, 130, 64, 3])


@pytest.mark.parametrize("bits,heads", [(2, (4, 8)), (3, (8, 8)), (4, (2, 16))])
def test_seeded_fp32_tables(bits, heads):
    wl = S.workload("c2", bits=bits, n_kv_heads=heads[0], n_q_heads=heads[1])
    hit = False
    for seed in (11, 12):
        lut_k = S.make_lut(bits, seed, 0, 0, fp16_exact=False)
        lut_v = S.make_lut(bits, seed, 0, 1, fp16_exact=False)
        hit |= _run_case(wl, lut_k, lut_v, 389, [200, 1, 64])
    assert hit or bits == 2      # with 2 interior signposts the rounding may move no code; wider tables must


def test_lut_load_rejects_signposts_outside_fp16():
    import paper_2401_18079_amd as K
    wl = S.workload("c1")
    lay = S.LayerInputs(wl)
    gc = K.KvqCache(wl.bits, 1, 1, 128, lay.k_side, wl.rope_base, 1024)
    bad = lay.lut_k.copy(); bad[-1] = 70000.0
    with pytest.raises(K.KvqError):
        K.kvq_lut_load(gc, bad, lay.lut_v, lay.s, lay.z, lay.lo, lay.hi)
