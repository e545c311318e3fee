"""Full-size parity: the benchmark workload (LLaMA-7B layer shape, context 131072, nuq3, 1 % outliers)
in the launch configuration bench.py times, checked against the oracle on sampled token windows.

The GPU cache is filled on the device from the counter-based generator.  For seeded windows of 128
tokens the same tokens are regenerated on the host, quantized and packed by the oracle at their true
positions, and compared bit for bit; scores are compared at those positions (the oracle evaluates
them from its own quantized tokens), and the Value mat-vec is compared with a probability vector that
is non-zero only on the sampled tokens, so the oracle needs no other token."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, matvec_close

pytestmark = pytest.mark.gpu

L = 131072 + 37          # ragged: the last 64-token block is partly filled
N_WINDOWS = 12
WIN = 128


def _check_fused_against_separate_calls(gc, q, scale, scores, Ln, cap):
    """The fused decode call at full size: the same scores bit for bit and the same output as softmax
    and Value mat-vec run as separate calls on those scores (whose parts the caller has tied to the
    oracle; at small sizes the fused call is compared with the oracle itself)."""
    import torch
    import paper_2401_18079_amd as K
    Hq = gc.c.n_q_heads
    probs = torch.zeros((Hq, cap), device="cuda")
    out = torch.zeros((Hq, 128), device="cuda")
    ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(Hq, cap), dtype=torch.uint8, device="cuda")
    K.kvq_softmax_f32(scores, probs, Ln, ws)
    K.kvq_pv_matvec(gc, probs, out)
    fscores = torch.zeros((Hq, cap), device="cuda")
    fout = torch.zeros((Hq, 128), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), scale, fscores, fout)
    assert torch.equal(fscores[:, :Ln], scores[:, :Ln])
    ok, worst = matvec_close(fout.cpu().numpy(), out.cpu().numpy(), rel=2e-5)
    assert ok, f"fused against separate calls: worst error / bound = {worst:.3f}"


def test_c2_full_context_sampled_parity():
    import torch
    import paper_2401_18079_amd as K
    import bench

    wl = S.workload("c2")
    st = Setup(wl)
    cap = ((L + 127) // 128) * 128
    gc, dg, _, _ = bench.build_cache(st, L, cap, K, torch)
    assert gc.status() == 0 and gc.n_tokens_k == L and gc.n_tokens_v == L

    rng = np.random.default_rng(wl.seed)
    starts = sorted(set([0, (L // WIN) * WIN] + [int(x) * WIN for x in rng.integers(1, L // WIN, N_WINDOWS - 2)]))
    H, D, bits = wl.n_kv_heads, wl.D, wl.bits
    nbytes = O.codes_bytes(bits, H, cap)
    ok_codes = np.zeros(nbytes, np.uint8)
    ov_codes = np.zeros(nbytes, np.uint8)
    o_sz = np.zeros((cap, 2), np.uint16)
    kcnt = np.zeros(cap, np.uint32)
    vcnt = np.zeros(cap, np.uint32)
    kidx, kval, vidx, vval = [], [], [], []
    sampled = []
    for t0 in starts:
        T = min(WIN, L - t0)
        sampled += list(range(t0, t0 + T))
        kc, cnt, idx, val = O.quantize_k(st.k(t0, T), bits, st.lut_k_stored, st.s, st.z, st.lo, st.hi)
        O._pack_k(ok_codes, bits, H, cap, t0, T, kc)
        kcnt[t0:t0 + T] = cnt; kidx.append(idx); kval.append(val)
        sz, vc, cnt, idx, val = O.quantize_v(st.v(t0, T), bits, st.lut_v_stored, st.k_side)
        O._pack_v(ov_codes, bits, H, cap, t0, T, vc)
        o_sz[t0:t0 + T] = sz
        vcnt[t0:t0 + T] = cnt; vidx.append(idx); vval.append(val)
    sampled = np.array(sampled)

    # ---- packed codes, scale/zero, sparse entries of the sampled tokens: bit exact ------------------
    gk = gc.k_codes.cpu().numpy(); gv = gc.v_codes.cpu().numpy()
    gsz = gc.v_sz.cpu().numpy().view(np.uint16).reshape(cap, 2)
    gkp = gc.k_ptr.cpu().numpy().view(np.uint32); gvp = gc.v_ptr.cpu().numpy().view(np.uint32)
    gki = gc.k_idx.cpu().numpy().view(np.uint16); gkv = gc.k_val.cpu().numpy().view(np.uint16)
    gvi = gc.v_idx.cpu().numpy().view(np.uint16); gvv = gc.v_val.cpu().numpy().view(np.uint16)
    chunk = 16 * bits
    for wi, t0 in enumerate(starts):
        T = min(WIN, L - t0)
        for h in range(H):
            for blk in range(t0 // 64, (t0 + T + 63) // 64):      # Key blocks of 64 tokens
                a = h * cap * chunk + blk * 64 * chunk
                full = (blk + 1) * 64 <= t0 + T
                if full:
                    assert np.array_equal(gk[a:a + 64 * chunk], ok_codes[a:a + 64 * chunk]), ("k_codes", t0, h, blk)
            for g in range(2):                                     # Value blocks of 64 token pairs
                a = (h * 2 + g) * (cap // 2) * chunk + (t0 // 128) * 64 * chunk
                if T == WIN:
                    assert np.array_equal(gv[a:a + 64 * chunk], ov_codes[a:a + 64 * chunk]), ("v_codes", t0, h, g)
        assert np.array_equal(gsz[t0:t0 + T], o_sz[t0:t0 + T])
        assert np.array_equal(np.diff(gkp[t0:t0 + T + 1].astype(np.int64)), kcnt[t0:t0 + T])
        assert np.array_equal(np.diff(gvp[t0:t0 + T + 1].astype(np.int64)), vcnt[t0:t0 + T])
        assert np.array_equal(gki[gkp[t0]:gkp[t0 + T]], kidx[wi]) and np.array_equal(gkv[gkp[t0]:gkp[t0 + T]], kval[wi])
        assert np.array_equal(gvi[gvp[t0]:gvp[t0 + T]], vidx[wi]) and np.array_equal(gvv[gvp[t0]:gvp[t0 + T]], vval[wi])
    # the ragged last window: compare its tokens code by code through the oracle's unpacker
    t0 = starts[-1]; T = L - t0
    a = np.zeros((T, D), np.uint8); b = np.zeros((T, D), np.uint8)
    O._unpack_k(gk, bits, H, cap, t0, T, a); O._unpack_k(ok_codes, bits, H, cap, t0, T, b)
    assert np.array_equal(a, b)
    O._unpack_v(gv, bits, H, cap, t0, T, a); O._unpack_v(ov_codes, bits, H, cap, t0, T, b)
    assert np.array_equal(a, b)

    # ---- scores at the sampled positions ---------------------------------------------------------------
    def ptr_of(cnt):
        p = np.zeros(cap + 1, np.uint32)
        np.cumsum(cnt, out=p[1:])
        return p
    okp, ovp = ptr_of(kcnt), ptr_of(vcnt)
    oki, okv = np.concatenate(kidx), np.concatenate(kval)
    ovi, ovv = np.concatenate(vidx), np.concatenate(vval)
    q = S.gen_q(wl, 0, 0)
    scale = np.float32(1.0 / np.sqrt(128.0))
    ref = np.zeros((wl.n_q_heads, L), np.float32)
    O._qk(ok_codes, bits, H, wl.n_q_heads, cap, L, st.lut_k_stored, O._as_bits(st.s), O._as_bits(st.z), okp,
          oki if oki.size else np.zeros(1, np.uint16), okv if okv.size else np.zeros(1, np.uint16),
          np.ascontiguousarray(q), float(scale), float(wl.rope_base), ref, L, 0, np.zeros(1, np.uint16))
    scores = torch.zeros((wl.n_q_heads, cap), device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), float(scale), scores)
    got = scores.cpu().numpy()
    ok, worst = matvec_close(got[:, sampled], ref[:, sampled])
    assert ok, f"scores: worst error / bound = {worst:.3f}"

    # ---- Value mat-vec with probabilities supported on the sampled tokens -----------------------------------
    p = np.zeros((wl.n_q_heads, L), np.float32)
    p[:, sampled] = O.softmax(np.ascontiguousarray(ref[:, sampled]))
    ref_out = np.zeros((wl.n_q_heads, 128), np.float32)
    O._pv(ov_codes, bits, H, wl.n_q_heads, cap, L, st.lut_v_stored, o_sz, ovp, ovi, ovv, p, L, ref_out, 0, np.zeros(1, np.uint16))
    pfull = torch.zeros((wl.n_q_heads, cap), device="cuda")
    pfull[:, :L] = torch.from_numpy(p).cuda()
    out = torch.zeros((wl.n_q_heads, 128), device="cuda")
    K.kvq_pv_matvec(gc, pfull, out)
    ok, worst = matvec_close(out.cpu().numpy(), ref_out)
    assert ok, f"outputs: worst error / bound = {worst:.3f}"

    # ---- a property that holds at any size: the Value mat-vec is linear in the probabilities -------------
    pa = torch.rand((wl.n_q_heads, cap), device="cuda") / L
    pb = torch.rand((wl.n_q_heads, cap), device="cuda") / L
    oa, ob, oab = (torch.zeros((wl.n_q_heads, 128), device="cuda") for _ in range(3))
    K.kvq_pv_matvec(gc, pa, oa); K.kvq_pv_matvec(gc, pb, ob); K.kvq_pv_matvec(gc, pa + pb, oab)
    assert torch.allclose(oab, oa + ob, rtol=1e-4, atol=1e-6)

    _check_fused_against_separate_calls(gc, q, float(scale), scores, Ln=L, cap=cap)


def test_c3_million_token_context_sampled_parity():
    """Configuration 3 at its full size (context 1,048,576 + a ragged tail, nuq4, 0.1 % outliers): every
    wavefront of the sparse kernels walks many sub-ranges here and positions reach 2^20, where the
    rotary angle needs its two-float reduction.  The reference is evaluated only on the sampled windows
    (the oracle's reconstruction and rotation, token by token), so the test stays within seconds."""
    Lc = (1 << 20) + 77
    _sampled_full_size_parity(S.workload("c3"), Lc, [0, (Lc // WIN) * WIN, (1 << 20) - WIN], n_random=5)


def test_c4_half_million_token_gqa_context_sampled_parity():
    """Configuration 4's sequence at its full size (32 query / 8 KV heads, context 524,288 + a ragged
    tail, nuq2, 1 % outliers, rotary base 500000): four query heads share every KV head's codes in the
    launch configuration the benchmark times for this shape."""
    Lc = (1 << 19) + 55
    _sampled_full_size_parity(S.workload("c4"), Lc, [0, (Lc // WIN) * WIN, (1 << 19) - WIN], n_random=4)


def test_c5_last_layer_million_token_context_sampled_parity():
    """One layer of configuration 5 at its full size (the last of the 32: its own look-up tables and
    per-channel constants; context 1,048,576 + a ragged tail, nuq3, 1 % outliers: eight times the
    benchmark workload's context, 32 tiles per workgroup of the dense kernels)."""
    Lc = (1 << 20) + 21
    _sampled_full_size_parity(S.workload("c5"), Lc, [0, (Lc // WIN) * WIN, (1 << 20) - WIN], n_random=4, layer=31)


def _sampled_full_size_parity(wl, Lc, fixed_starts, n_random, layer=0):
    import torch
    import paper_2401_18079_amd as K
    import bench

    st = Setup(wl, layer)
    cap = ((Lc + 127) // 128) * 128
    gc, dg, _, _ = bench.build_cache(st, Lc, cap, K, torch)
    assert gc.status() == 0 and gc.n_tokens_k == Lc and gc.n_tokens_v == Lc

    H, Hq, D, bits = wl.n_kv_heads, wl.n_q_heads, wl.D, wl.bits
    rng = np.random.default_rng(wl.seed + 3)
    starts = sorted(set(list(fixed_starts) + [int(x) * WIN for x in rng.integers(1, Lc // WIN, n_random)]))
    gkp = gc.k_ptr.cpu().numpy().view(np.uint32); gvp = gc.v_ptr.cpu().numpy().view(np.uint32)
    gsz = gc.v_sz.cpu().numpy().view(np.uint16).reshape(cap, 2)
    q = S.gen_q(wl, 0, 0)
    scale = np.float32(1.0 / np.sqrt(128.0))
    scores = torch.zeros((Hq, cap), device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q).cuda(), float(scale), scores)
    sampled, ref_cols, vhat_rows = [], [], []
    gk, gv = gc.k_codes.cpu().numpy(), gc.v_codes.cpu().numpy()
    for t0 in starts:
        T = min(WIN, Lc - t0)
        # a small oracle cache that holds just this window, at capacity 128, for quantization ...
        kc, kcnt, kidx, kval = O.quantize_k(st.k(t0, T), bits, st.lut_k_stored, st.s, st.z, st.lo, st.hi)
        sz, vc, vcnt, vidx, vval = O.quantize_v(st.v(t0, T), bits, st.lut_v_stored, st.k_side)
        # ... compared bit for bit with what the device stored at the true positions
        a = np.zeros((T, D), np.uint8)
        O._unpack_k(gk, bits, H, cap, t0, T, a)
        assert np.array_equal(a, kc), ("k codes", t0)
        O._unpack_v(gv, bits, H, cap, t0, T, a)
        assert np.array_equal(a, vc), ("v codes", t0)
        assert np.array_equal(gsz[t0:t0 + T], sz)
        assert np.array_equal(np.diff(gkp[t0:t0 + T + 1].astype(np.int64)), kcnt)
        assert np.array_equal(np.diff(gvp[t0:t0 + T + 1].astype(np.int64)), vcnt)
        assert np.array_equal(gc.k_idx[int(gkp[t0]):int(gkp[t0 + T])].cpu().numpy().view(np.uint16), kidx)
        assert np.array_equal(gc.k_val[int(gkp[t0]):int(gkp[t0 + T])].cpu().numpy().view(np.uint16), kval)
        assert np.array_equal(gc.v_idx[int(gvp[t0]):int(gvp[t0 + T])].cpu().numpy().view(np.uint16), vidx)
        assert np.array_equal(gc.v_val[int(gvp[t0]):int(gvp[t0 + T])].cpu().numpy().view(np.uint16), vval)
        # reference scores of the window: the oracle's reconstruction and rotation at the true positions
        win = O.OracleCache(bits, H, Hq, 128, st.k_side, wl.rope_base, st.lut_k_stored, st.lut_v_stored, st.s, st.z, st.lo, st.hi)
        win.append_k(st.k(t0, T)); win.append_v(st.v(t0, T))
        khat, vhat = win.reconstruct_k(0, T), win.reconstruct_v(0, T)
        g = Hq // H
        col = np.zeros((Hq, T))
        for t in range(T):
            for hk in range(H):
                krot = O.rope(khat[t, hk * 128:(hk + 1) * 128], t0 + t, wl.rope_base)
                for j in range(g):
                    col[hk * g + j, t] = float(scale) * np.dot(q[hk * g + j].astype(np.float64), krot)
        sampled += list(range(t0, t0 + T)); ref_cols.append(col); vhat_rows.append(vhat)
    sampled = np.array(sampled)
    ref = np.concatenate(ref_cols, axis=1)
    got = scores.cpu().numpy()[:, sampled]
    # the row RMS of the bound is taken over the sampled columns only
    ok, worst = matvec_close(got, ref.astype(np.float32))
    assert ok, f"scores: worst error / bound = {worst:.3f}"

    # Value mat-vec with probabilities supported on the sampled tokens
    vhat = np.concatenate(vhat_rows, axis=0)                       # [n_sampled][D]
    psub = O.softmax(np.ascontiguousarray(ref.astype(np.float32)))
    g = Hq // H
    ref_out = np.stack([psub[h].astype(np.float64) @ vhat[:, (h // g) * 128:(h // g + 1) * 128] for h in range(Hq)])
    pfull = torch.zeros((Hq, cap), device="cuda")
    pfull[:, torch.from_numpy(sampled).cuda()] = torch.from_numpy(psub).cuda()
    out = torch.zeros((Hq, 128), device="cuda")
    K.kvq_pv_matvec(gc, pfull, out)
    ok, worst = matvec_close(out.cpu().numpy(), ref_out.astype(np.float32))
    assert ok, f"outputs: worst error / bound = {worst:.3f}"
    _check_fused_against_separate_calls(gc, q, float(scale), scores, Ln=Lc, cap=cap)


def test_c2_full_context_constant_value_rows_closed_form():
    """A closed form that needs no oracle and covers every token of the full-size workload.  Every
    Value vector is constant, v[n][:] = c_n.  Then (paper Sec. 3.4/3.6 with the tie rules of the
    per-token selection) the first 2*k_side channels are the outliers, zero-point = c_n, scale = 1,
    every code is the signpost l0 nearest to zero, an outlier's residual is -l0, and the de-quantised
    row is c_n on the outlier channels and c_n + l0 elsewhere.  So for any weights w:
        out[h][c] = sum_n w[h][n] * c_n  (+ l0 * sum_n w[h][n]  on the other channels),
    which is checked for kvq_pv_matvec with given probabilities and for the fused call with the
    softmax of the scores it returns (evaluated on the host in fp64)."""
    import torch
    import paper_2401_18079_amd as K
    from kvq_synth.device import DeviceGen

    wl = S.workload("c2")
    st = Setup(wl)
    Lc = 131072 + 37
    cap = ((Lc + 127) // 128) * 128
    gc = st.gpu_cache(cap)
    dg = DeviceGen(wl, st.layer, st.kprof, st.vprof)
    n_all = torch.arange(Lc, device="cuda")
    c_all = ((n_all % 7) - 3).to(torch.float16)                     # c_n in {-3, ..., 3}
    t0 = 0
    while t0 < Lc:
        T = min(4096, Lc - t0)
        K.kvq_quantize_append_k(gc, dg.k(t0, T))
        K.kvq_quantize_append_v(gc, c_all[t0:t0 + T, None].expand(T, wl.D).contiguous())
        t0 += T
    torch.cuda.synchronize()
    assert gc.status() == 0 and gc.n_tokens_v == Lc

    lut_v = np.asarray(st.lut_v_stored, dtype=np.float32)
    l0 = float(lut_v[int(np.argmin(np.abs(lut_v)))])                # first minimum: ties to the smaller index
    n_out = 2 * st.k_side
    c_host = c_all.float().cpu().numpy().astype(np.float64)
    # what the append stored: outliers are channels 0 .. 2*k_side-1 of every token, residual -l0
    vp = gc.v_ptr.cpu().numpy().view(np.uint32)[:Lc + 1].astype(np.int64)
    assert np.array_equal(np.diff(vp), np.full(Lc, n_out))
    for n in (0, 1, 4095, 4096, Lc - 1):
        idx = gc.v_idx[int(vp[n]):int(vp[n + 1])].cpu().numpy().view(np.uint16)
        val = gc.v_val[int(vp[n]):int(vp[n + 1])].cpu().numpy().view(np.float16)
        assert np.array_equal(idx, np.arange(n_out, dtype=np.uint16))
        assert np.all(val.astype(np.float32) == np.float32(-l0))

    def expected(w):                                                 # w: [Hq][Lc] float64
        base = w @ c_host                                            # [Hq]
        out = np.repeat(base[:, None], 128, axis=1) + l0 * w.sum(axis=1)[:, None]
        g = wl.n_q_heads // wl.n_kv_heads
        for h in range(wl.n_q_heads):                                # outlier channels all lie in KV head 0
            if h // g == 0:
                out[h, :min(n_out, 128)] = base[h]
        return out

    assert n_out <= 128
    # (1) the Value mat-vec alone, with probabilities that vary over the whole context
    p = torch.softmax(torch.randn((wl.n_q_heads, Lc), device="cuda", generator=torch.Generator("cuda").manual_seed(5)) * 2.0, dim=1)
    pfull = torch.zeros((wl.n_q_heads, cap), device="cuda")
    pfull[:, :Lc] = p
    out = torch.zeros((wl.n_q_heads, 128), device="cuda")
    K.kvq_pv_matvec(gc, pfull, out)
    ok, worst = matvec_close(out.cpu().numpy(), expected(p.double().cpu().numpy()))
    assert ok, f"pv closed form: worst error / bound = {worst:.3f}"
    # (2) the fused call: its weights are the softmax of the scores it leaves behind
    q = S.gen_q(wl, 0, 0)
    scores = torch.zeros((wl.n_q_heads, cap), device="cuda")
    K.kvq_attention_decode(gc, torch.from_numpy(q).cuda(), 1.0 / np.sqrt(128.0), scores, out)
    x = scores[:, :Lc].double().cpu().numpy()
    w = np.exp(x - x.max(axis=1, keepdims=True))
    w /= w.sum(axis=1, keepdims=True)
    ok, worst = matvec_close(out.cpu().numpy(), expected(w))
    assert ok, f"fused closed form: worst error / bound = {worst:.3f}"


def test_c2_full_context_constant_keys_closed_form():
    """Every Key equals its channel's zero-point, so every code is the signpost l0 nearest to zero,
    no element is an outlier, and the de-quantised Key is the same vector k = s*l0 + z at every
    position.  The score of token n is then the closed form of the rotary product (paper App. "RoPE
    Equation", half-split pairs):
        scale * sum_i (q_i k_i + q_{i+64} k_{i+64}) cos(n theta_i) + (q_{i+64} k_i - q_i k_{i+64}) sin(n theta_i),
    evaluated here in fp64 for every token of the full context (no oracle involved)."""
    import torch
    import paper_2401_18079_amd as K

    wl = S.workload("c2")
    st = Setup(wl)
    Lc = 131072 + 37
    cap = ((Lc + 127) // 128) * 128
    gc = st.gpu_cache(cap)
    z16 = np.asarray(st.z, dtype=np.float16)
    row = torch.from_numpy(z16).cuda()
    t0 = 0
    while t0 < Lc:
        T = min(4096, Lc - t0)
        K.kvq_quantize_append_k(gc, row[None, :].expand(T, wl.D).contiguous())
        t0 += T
    torch.cuda.synchronize()
    assert gc.status() == 0 and int(gc.k_ptr[Lc].item()) == 0           # not a single outlier

    lut_k = np.asarray(st.lut_k_stored, dtype=np.float32)
    l0 = np.float32(lut_k[int(np.argmin(np.abs(lut_k)))])
    s32 = np.asarray(st.s, dtype=np.float16).astype(np.float32)
    # fmaf(s, l0, z): the exact sum rounded once to fp32
    khat = np.float32(s32.astype(np.float64) * np.float64(l0) + z16.astype(np.float64)).astype(np.float64)
    q = S.gen_q(wl, 0, 0).astype(np.float64)
    scale = 1.0 / np.sqrt(128.0)
    n = np.arange(Lc, dtype=np.float64)
    theta = wl.rope_base ** (-2.0 * np.arange(64) / 128.0)
    ang = n[:, None] * theta[None, :]
    cs, sn = np.cos(ang), np.sin(ang)                                   # [Lc][64]
    g = wl.n_q_heads // wl.n_kv_heads
    ref = np.zeros((wl.n_q_heads, Lc))
    for h in range(wl.n_q_heads):
        k = khat[(h // g) * 128:(h // g + 1) * 128]
        A = q[h, :64] * k[:64] + q[h, 64:] * k[64:]
        B = q[h, 64:] * k[:64] - q[h, :64] * k[64:]
        ref[h] = scale * (cs @ A + sn @ B)
    scores = torch.zeros((wl.n_q_heads, cap), device="cuda")
    K.kvq_qk_matvec(gc, torch.from_numpy(q.astype(np.float32)).cuda(), scale, scores)
    ok, worst = matvec_close(scores[:, :Lc].cpu().numpy(), ref)
    assert ok, f"scores closed form: worst error / bound = {worst:.3f}"
