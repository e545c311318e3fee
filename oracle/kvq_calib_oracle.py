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
