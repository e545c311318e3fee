"""CPU oracle of the offline derivation of the non-uniform datatype (paper Sec. 3.3, Eq. (1), and the
appendix on per-channel scaling: the signposts minimise  sum_i F_ii s_i^2 (A_norm,i - Q(A_norm,i))^2
over the normalised calibration activations, "using a k-means solver").

TEST INFRASTRUCTURE ONLY: imported by tests/; the GPU library never imports or calls it.

The solver is Lloyd's algorithm in one dimension, written out step by step in numpy: assignment of
every element to its nearest signpost, then every signpost moves to the weighted mean of its
elements.  Where the paper is silent this file takes these readings (the GPU path takes the same
ones, in its own code):
  * weights  w_i = F_ii * s_i^2  are an input (one number per element);
  * the initial signposts are an input; the number of iterations is fixed by the caller;
  * nearest = smallest |x - c_j| evaluated in fp32, ties to the smaller index (as for quantization);
  * sums are taken in fp64 (w*x of two fp32 numbers is exact in fp64); a signpost is rounded to fp32
    after every update; a signpost whose elements have total weight zero stays where it is;
  * the result is returned sorted.
"""
from __future__ import annotations

import numpy as np


def nearest(x, c):
    """Index of the nearest signpost for every x: fp32 distances, first minimum wins."""
    x = np.asarray(x, dtype=np.float32)
    c = np.asarray(c, dtype=np.float32)
    best = np.zeros(x.shape, dtype=np.int64)
    bestd = np.abs(x - c[0])                       # fp32 - fp32 -> fp32
    for j in range(1, c.size):
        d = np.abs(x - c[j])
        closer = d < bestd
        best = np.where(closer, j, best)
        bestd = np.where(closer, d, bestd)
    return best


def lloyd_step(x, w, c):
    """One iteration: returns the updated signposts (fp32) for signposts c."""
    x = np.asarray(x, dtype=np.float32)
    w = np.asarray(w, dtype=np.float32)
    c = np.asarray(c, dtype=np.float32).copy()
    idx = nearest(x, c)
    w64, x64 = w.astype(np.float64), x.astype(np.float64)
    for j in range(c.size):
        m = idx == j
        sw = float(np.sum(w64[m]))
        if sw > 0.0:
            c[j] = np.float32(float(np.sum(w64[m] * x64[m])) / sw)
    return c


def nuq_signposts(x_norm, w, c_init, iters):
    """Eq. (1) with the s_i^2 weighting folded into w: `iters` Lloyd iterations from c_init, sorted."""
    c = np.asarray(c_init, dtype=np.float32).copy()
    for _ in range(int(iters)):
        c = lloyd_step(x_norm, w, c)
    return np.sort(c)


def objective(x_norm, w, c):
    """sum_i w_i (x_i - Q(x_i))^2 in fp64, Q = nearest signpost."""
    x = np.asarray(x_norm, dtype=np.float32)
    c = np.asarray(c, dtype=np.float32)
    q = c[nearest(x, c)].astype(np.float64)
    return float(np.sum(np.asarray(w, dtype=np.float64) * (x.astype(np.float64) - q) ** 2))


def key_channel_constants(x16, outlier_fraction):
    """Offline per-channel calibration of the Keys (paper Sec. 3.6 and the appendix on offline
    calibration: per-channel outlier thresholds, scaling factors and zero-points come from a
    calibration set; Sec. 3.4: the thresholds isolate a fixed fraction of each channel as outliers).

    x16: fp16 calibration Keys [T][D] (pre-RoPE).  Readings where the paper gives no formula:
      * k = floor(outlier_fraction / 2 * T + 1/2) elements per side and channel;
      * with the channel's values sorted ascending as xs: lower threshold xs[k-1], upper threshold
        xs[T-k] (the k-th smallest / largest value), and the range that is normalised to [-1, 1] is
        [xs[k], xs[T-k-1]], the values strictly inside; k = 0: thresholds -65504 / +65504, range
        [xs[0], xs[T-1]];
      * zero-point = mid-range, scale = half-range, each computed in fp32 and rounded to fp16;
        a scale that is not positive becomes 1; zeros are returned as +0.
    Returns fp16 arrays (s, z, lo, hi) of shape [D]."""
    x = np.asarray(x16, dtype=np.float16).astype(np.float32)
    T, D = x.shape
    k = int(np.floor(float(outlier_fraction) / 2.0 * T + 0.5))
    assert 2 * k < T
    s = np.zeros(D, np.float16); z = np.zeros(D, np.float16)
    lo = np.zeros(D, np.float16); hi = np.zeros(D, np.float16)
    for c in range(D):
        xs = np.sort(x[:, c], kind="stable")
        if k > 0:
            lo[c], hi[c] = np.float16(xs[k - 1]), np.float16(xs[T - k])
            a, b = xs[k], xs[T - k - 1]
        else:
            lo[c], hi[c] = np.float16(-65504.0), np.float16(65504.0)
            a, b = xs[0], xs[T - 1]
        z[c] = np.float16((np.float32(b) + np.float32(a)) * np.float32(0.5))
        sc = np.float16((np.float32(b) - np.float32(a)) * np.float32(0.5))
        s[c] = sc if np.float32(sc) > 0 else np.float16(1.0)
    # a zero is returned as +0 whatever the signs of the zeros in the data (no comparison or sum
    # downstream can tell the two apart)
    pz = np.float16(0.0)
    return s, z + pz, lo + pz, hi + pz
