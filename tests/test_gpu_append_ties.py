"""GPU parity for the Value append on vectors full of equal elements: the per-token top-k / bottom-k
outlier choice must break ties exactly like the oracle (lower index first, largest side chosen before
the smallest side), whichever internal route the kernel takes (both thresholds found together, ties
straddling one or both thresholds, thresholds that coincide)."""
import numpy as np
import pytest

import kvq_synth as S
from oracle import kvq_oracle as O
from kvq_testlib import Setup, compare_caches, matvec_close

pytestmark = pytest.mark.gpu


def _tie_vectors(D, k, rng):
    rows = []
    rows.append(np.zeros(D))                                             # all equal (zero range)
    rows.append(rng.choice([-1.0, 0.0, 1.0], size=D))                    # three values: ties on both sides
    rows.append(np.round(rng.standard_normal(D), 1))                     # coarse grid: many ties
    x = np.full(D, -2.0); x[rng.choice(D, D // 3, replace=False)] = rng.uniform(1, 50, D // 3)
    rows.append(x)                                                       # distinct top, tied bottom
    rows.append(-x)                                                      # tied top, distinct bottom
    rows.append(np.full(D, 7.5))                                         # all equal, non-zero
    x = np.full(D, 3.0); x[rng.choice(D, D // 2, replace=False)] = -3.0
    rows.append(x)                                                       # two values
    x = rng.choice([0.0, -0.0, 1e-3, -1e-3], size=D)
    rows.append(x)                                                       # signed zeros among small values
    x = np.full(D, 0.25); x[rng.choice(D, k, replace=False)] = rng.uniform(5, 9, k)
    rows.append(x)                                                       # exactly k large ones
    x = np.full(D, 0.25); x[rng.choice(D, k - 1, replace=False)] = rng.uniform(5, 9, k - 1)
    rows.append(x)                                                       # k-1 large ones: thresholds coincide
    rows.append(rng.standard_normal(D))                                  # ordinary
    rows.append(np.repeat(np.arange(D // 2), 2) / 64.0)                  # every value twice, ascending
    x = np.full(D, 1.0); x[:k] = 2.0; x[-k:] = 0.5
    rows.append(x)                                                       # outliers exactly fill both sides
    x = np.full(D, 1.0); x[: k + 3] = 2.0; x[-(k + 3):] = 0.5
    rows.append(x)                                                       # three too many on both sides
    return np.stack(rows).astype(np.float16)


@pytest.mark.parametrize("heads,bits", [(4, 3), (32, 3), (16, 4), (2, 2)])
def test_value_append_ties(heads, bits):
    import torch
    import paper_2401_18079_amd as K
    wl = S.workload("c2", n_kv_heads=heads, n_q_heads=heads, bits=bits)
    st = Setup(wl)
    assert st.k_side >= 1
    rng = np.random.default_rng(100 + heads)
    v = _tie_vectors(wl.D, st.k_side, rng)
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
