"""GPU parity for the Value append on vectors full of equal elements: the per-token top-k / bottom-k
outlier choice must break ties exactly like the oracle (lower index first, largest side chosen before
the smallest side), whichever internal route the kernel takes (both thresholds found together, ties
straddling one or both thresholds, thresholds that coincide)."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close, tie_vectors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("heads,bits", [(4, 3), (32, 3), (16, 4), (2, 2)])
def test_value_append_ties(heads, bits):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=heads, n_q_heads=heads, bits=bits)
    st = Setup(wl)
    assert st.k_side >= 1
    rng = np.random.default_rng(100 + heads)
    v = tie_vectors(wl.D, st.k_side, rng)
    v = np.concatenate([v, v[::-1], v[rng.permutation(len(v))]])         # both pair parities see every row
    T = len(v)
    k = st.k(0, T)
    cap = 128
    oc, gc = st.oracle_cache(cap), st.gpu_cache(cap)
    t0 = 0
    for chunk in [1, 1, 2, 5, 1, 9, 3]:
        chunk = min(chunk, T - t0)
        if chunk <= 0:
            break
        oc.append_k(k[t0:t0 + chunk]); oc.append_v(v[t0:t0 + chunk])
        K.kvq_quantize_append_k(gc, torch.from_numpy(k[t0:t0 + chunk]).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v[t0:t0 + chunk]).cuda())
        t0 += chunk
    while t0 < T:                                                        # the rest one token at a time
        oc.append_k(k[t0:t0 + 1]); oc.append_v(v[t0:t0 + 1])
        K.kvq_quantize_append_k(gc, torch.from_numpy(k[t0:t0 + 1]).cuda())
        K.kvq_quantize_append_v(gc, torch.from_numpy(v[t0:t0 + 1]).cuda())
        t0 += 1
    torch.cuda.synchronize()
    assert gc.status() == 0
    bad = compare_caches(oc, gc)
    assert not bad, bad
    p = O.softmax(rng.standard_normal((heads, T)))
    out = torch.empty((heads, 128), device="cuda")
    K.kvq_pv_matvec(gc, torch.from_numpy(p.astype(np.float32)).cuda(), out)
    ok, worst = matvec_close(out.cpu().numpy(), oc.pv(p.astype(np.float32)))
    assert ok, f"pv worst error / bound = {worst:.3f}"
