"""Shared helpers of the GPU parity tests: build the same synthetic cache through the CPU oracle and
through the HIP library (each with its own code), and the tolerance used for mat-vec results."""
import numpy as np

import kvq_synth as S
from oracle import kvq_oracle as O

REL_TOL = 1e-3      # spec tolerance: 1e-3 relative, fp32 accumulation


def matvec_close(got, ref, rel=REL_TOL):
    """|got - ref| <= rel*|ref| + rel*rms(ref) per row (scores cancel to ~0, so a purely relative
    test is ill-posed; the absolute floor is rel times the row's RMS)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    err = np.abs(got - ref)
    bound = rel * np.abs(ref) + rel * rms
    worst = float(np.max(err / np.maximum(bound, 1e-300)))
    return bool(np.all(err <= bound)), worst


class Setup(S.LayerInputs):
    """A synthetic layer's inputs plus the two caches under comparison."""

    def __init__(self, wl, layer=0):
        super().__init__(wl, layer)
        # the signposts as a cache stores them (fp16 numbers), for tests that call the oracle's
        # element-level functions directly; the caches below are handed the tables as drawn
        self.lut_k_stored, self.lut_v_stored = O.store_lut(self.lut_k), O.store_lut(self.lut_v)

    def oracle_cache(self, cap):
        wl = self.wl
        return O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, self.k_side, wl.rope_base, self.lut_k,
                             self.lut_v, self.s, self.z, self.lo, self.hi, cap_nnz_k=self.cap_nnz_k(cap))

    def gpu_cache(self, cap, max_append=4096):
        import paper_2401_18079_amd as K
        wl = self.wl
        c = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, self.k_side, wl.rope_base, self.cap_nnz_k(cap),
                       max_append=max_append)
        K.kvq_lut_load(c, self.lut_k, self.lut_v, self.s, self.z, self.lo, self.hi)
        return c


def fill_both(setup: Setup, oc, gc, L, chunks, seq=0):
    """Append tokens [0, L) to both caches in the given chunk sizes (cycled)."""
    import torch
    import paper_2401_18079_amd as K
    t0, i = 0, 0
    while t0 < L:
        T = min(chunks[i % len(chunks)], L - t0)
        k, v = setup.k(t0, T, seq), setup.v(t0, T, seq)
        if oc is not None:
            oc.append_k(k)
            oc.append_v(v)
        if gc is not None:
            K.kvq_quantize_append_k(gc, torch.from_numpy(k).cuda())
            K.kvq_quantize_append_v(gc, torch.from_numpy(v).cuda())
        t0 += T
        i += 1


def compare_caches(oc, gc):
    """Bit-exact comparison of every stored array.  Returns a list of mismatch descriptions."""
    bad = []
    L = oc.n_k

    def chk(name, a, b):
        a = np.asarray(a); b = np.asarray(b)
        if a.shape != b.shape or not np.array_equal(a, b):
            n = int(np.sum(a != b)) if a.shape == b.shape else -1
            first = int(np.nonzero(a != b)[0][0]) if n > 0 else -1
            bad.append(f"{name}: {n} mismatches, first at {first}")

    g = lambda t: t.cpu().numpy()
    chk("k_codes", oc.k_codes, g(gc.k_codes))
    chk("v_codes", oc.v_codes, g(gc.v_codes))
    chk("v_sz", oc.v_sz.reshape(-1)[:2 * L], g(gc.v_sz).view(np.uint16)[:2 * L])
    chk("k_ptr", oc.k_ptr[:L + 1], g(gc.k_ptr).view(np.uint32)[:L + 1])
    chk("v_ptr", oc.v_ptr[:L + 1], g(gc.v_ptr).view(np.uint32)[:L + 1])
    nk, nv = int(oc.k_ptr[L]), int(oc.v_ptr[L])
    (k_idx, k_val), (v_idx, v_val) = gc.sparse_entries("k", nk), gc.sparse_entries("v", nv)   # flat or blocked
    chk("k_idx", oc.k_idx[:nk], g(k_idx).view(np.uint16))
    chk("k_val", oc.k_val[:nk], g(k_val).view(np.uint16))
    chk("v_idx", oc.v_idx[:nv], g(v_idx).view(np.uint16))
    chk("v_val", oc.v_val[:nv], g(v_val).view(np.uint16))
    return bad


def tie_vectors(D, k, rng):
    """Value vectors full of equal elements, one row per way the top-k / bottom-k thresholds can meet ties
    (k = outliers per side)."""
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
