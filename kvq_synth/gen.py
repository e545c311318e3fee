"""Counter-based synthetic activations shaped like long-context LLaMA decode.

Every element is a pure function of (seed, tensor, layer, sequence, token, channel), built
from integer hashing plus single correctly-rounded fp32 operations, so any slice of any
tensor can be regenerated independently and identically anywhere.

Distributional structure (what the paper reports about real KV activations, its Fig. on
activation distributions and the dynamic-range appendix): pre-RoPE Keys have a few fixed
channels of much larger magnitude and per-channel offsets; Values have milder channel and
token scale variation; in both, ~99 % of a vector sits in a small part of its range, with a
few far outliers.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

SEED_BASE = 20240118

T_K, T_V, T_Q, T_KCAL, T_AUX = 1, 2, 3, 4, 5

_U64 = np.uint64
_M1 = _U64(0x9E3779B97F4A7C15)
_M2 = _U64(0xBF58476D1CE4E5B9)
_M3 = _U64(0x94D049BB133111EB)
_INV_STD = np.float32(1.0 / 37837.227)  # 1/std of a sum of four uniform 16-bit integers


@dataclasses.dataclass(frozen=True)
class Workload:
    """One row of the benchmark configuration list (shapes only, no data)."""
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int
    bits: int
    outlier_fraction: float
    rope_base: float
    batch: int
    n_layers: int
    key_profile: str          # "spiky8" (8 channels x20) or "student_t" (heavy-tailed scales)
    seed: int

    @property
    def D(self) -> int:
        return self.n_kv_heads * self.head_dim


WORKLOADS = {
    "c1": Workload("c1", 1, 1, 128, 4096, 3, 0.01, 10000.0, 1, 1, "spiky8", SEED_BASE + 0),
    "c2": Workload("c2", 32, 32, 128, 131072, 3, 0.01, 10000.0, 1, 1, "student_t", SEED_BASE + 1),
    "c3": Workload("c3", 32, 32, 128, 1048576, 4, 0.001, 10000.0, 1, 1, "student_t", SEED_BASE + 2),
    "c4": Workload("c4", 32, 8, 128, 524288, 2, 0.01, 500000.0, 8, 1, "student_t", SEED_BASE + 3),
    "c5": Workload("c5", 32, 32, 128, 1048576, 3, 0.01, 10000.0, 1, 32, "student_t", SEED_BASE + 4),
}


def workload(name: str, **overrides) -> Workload:
    return dataclasses.replace(WORKLOADS[name], **overrides)


def k_side_from_fraction(p: float, D: int) -> int:
    """Outliers kept per side of a D-vector for outlier fraction p (symmetric split)."""
    if p <= 0.0:
        return 0
    return max(1, int(math.floor(p * D / 2.0 + 0.5)))


def splitmix64(x):
    """SplitMix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (np.asarray(x, dtype=_U64) + _M1).astype(_U64)
        z = ((z ^ (z >> _U64(30))) * _M2).astype(_U64)
        z = ((z ^ (z >> _U64(27))) * _M3).astype(_U64)
        return (z ^ (z >> _U64(31))).astype(_U64)


def hash_grid(seed: int, tensor_id: int, layer: int, seq: int, tokens, channels):
    """64-bit hash for every (token, channel) pair; tokens < 2^24, channels < 2^16."""
    tokens = np.asarray(tokens, dtype=_U64).reshape(-1, 1)
    channels = np.asarray(channels, dtype=_U64).reshape(1, -1)
    key = (_U64(seed) ^ (_U64(tensor_id) << _U64(56)) ^ (_U64(layer) << _U64(48))
           ^ (_U64(seq) << _U64(40)))
    return splitmix64(key ^ (tokens << _U64(16)) ^ channels)


def normalish(h):
    """Unit-variance bell-shaped fp32 from a 64-bit hash (sum of its four 16-bit fields)."""
    m = _U64(0xFFFF)
    s = (h & m) + ((h >> _U64(16)) & m) + ((h >> _U64(32)) & m) + ((h >> _U64(48)) & m)
    return (s.astype(np.int64) - 131070).astype(np.float32) * _INV_STD


def _spiked(h):
    """normalish(h), multiplied by 6 for one element in 128 (far outliers)."""
    g = normalish(h)
    spike = np.where((splitmix64(h) & _U64(127)) == 0, np.float32(6.0), np.float32(1.0))
    return (g * spike).astype(np.float32)


def _vec_normal(seed, tensor_id, layer, n, salt):
    """n fp32 normal-ish draws for per-channel / per-token parameters."""
    h = hash_grid(seed, tensor_id, layer, 0xFF, [salt], np.arange(n))
    return normalish(h).reshape(-1)


def key_channel_profile(w: Workload, layer: int = 0):
    """Per-channel magnitude a_c and offset mu_c (fp32 [D]) of the synthetic Keys."""
    D = w.D
    seed = w.seed
    if w.key_profile == "spiky8":
        a = np.ones(D, dtype=np.float32)
        order = np.argsort(splitmix64(np.arange(D, dtype=_U64) ^ _U64(seed + 77 + layer)), kind="stable")
        a[order[:8]] = 20.0
        mu = (0.25 * _vec_normal(seed, T_AUX, layer, D, 2) * a).astype(np.float32)
        return a, mu
    # Student-t (nu=4) magnitudes: z / sqrt(chi2_4/4), floored at 0.05.
    z = _vec_normal(seed, T_AUX, layer, D, 3).astype(np.float64)
    chi = sum(_vec_normal(seed, T_AUX, layer, D, 4 + j).astype(np.float64) ** 2 for j in range(4))
    a = np.maximum(np.abs(z / np.sqrt(np.maximum(chi, 1e-3) / 4.0)), 0.05).astype(np.float32)
    mu = (0.5 * _vec_normal(seed, T_AUX, layer, D, 9) * a).astype(np.float32)
    return a, mu


def value_channel_profile(w: Workload, layer: int = 0):
    """Mild per-channel magnitude and offset (fp32 [D]) of the synthetic Values."""
    D = w.D
    a = np.exp(0.35 * _vec_normal(w.seed, T_AUX, layer, D, 12).astype(np.float64)).astype(np.float32)
    mu = (0.25 * _vec_normal(w.seed, T_AUX, layer, D, 13) * a).astype(np.float32)
    return a, mu


def value_token_scale(w: Workload, layer: int, seq: int, t0: int, T: int):
    """Per-token Value magnitude sigma_t = exp(0.5 g) (fp32 [T])."""
    h = hash_grid(w.seed, T_AUX, layer, seq, np.arange(t0, t0 + T), [0xFFFF])
    return np.exp(0.5 * normalish(h).reshape(-1).astype(np.float64)).astype(np.float32)


def gen_k(w: Workload, layer: int, seq: int, t0: int, T: int, profile=None, tensor_id: int = T_K):
    """Pre-RoPE Key activations for tokens [t0, t0+T): float16 [T][D]."""
    a, mu = profile if profile is not None else key_channel_profile(w, layer)
    h = hash_grid(w.seed, tensor_id, layer, seq, np.arange(t0, t0 + T), np.arange(w.D))
    g = _spiked(h)
    x = (g * a[None, :]).astype(np.float32) + mu[None, :]
    return x.astype(np.float32).astype(np.float16)


def gen_v(w: Workload, layer: int, seq: int, t0: int, T: int, profile=None):
    """Value activations for tokens [t0, t0+T): float16 [T][D]."""
    a, mu = profile if profile is not None else value_channel_profile(w, layer)
    sig = value_token_scale(w, layer, seq, t0, T)
    h = hash_grid(w.seed, T_V, layer, seq, np.arange(t0, t0 + T), np.arange(w.D))
    g = _spiked(h)
    u = (g * sig[:, None]).astype(np.float32)
    x = (u * a[None, :]).astype(np.float32) + mu[None, :]
    return x.astype(np.float32).astype(np.float16)


def gen_q(w: Workload, layer: int, seq: int, step: int = 0):
    """Query for one decode step, already position-rotated by the caller's model: fp32 [H_q][d].

    A rotation of an isotropic Gaussian vector is again isotropic Gaussian, so the rotated
    query is drawn directly."""
    h = hash_grid(w.seed, T_Q, layer, seq, np.arange(w.n_q_heads) + step * 256, np.arange(w.head_dim))
    return normalish(h).astype(np.float32)


def gen_probs_logits(w: Workload, layer: int, seq: int, L: int, temperature: float = 1.5):
    """Stand-alone attention logits fp32 [H_q][L] (for exercising softmax / PV on their own)."""
    h = hash_grid(w.seed, T_AUX, layer, seq, np.arange(w.n_q_heads) + 4096, np.arange(L) & 0xFFFF)
    h = splitmix64(h ^ (np.arange(L, dtype=_U64)[None, :] >> _U64(16)))
    return (normalish(h) * np.float32(temperature)).astype(np.float32)


def make_lut(bits: int, seed: int, layer: int, which: int, fp16_exact=None):
    """2^bits sorted signposts in [-1, 1] as fp32, adjacent gaps >= 2^-7 (also after rounding to fp16).

    The outermost signposts are pinned to -1 and +1 (a normalised vector always touches both
    ends of its range); the interior ones are seeded uniform draws.  A k-means solver returns
    fp32 signposts that are not fp16 numbers, and a cache stores fp16 signposts, so about one
    table in three (chosen by the seed; `fp16_exact` overrides) keeps its fp32 draws and the rest
    are fp16 numbers already."""
    n = 1 << bits
    if fp16_exact is None:
        pick = splitmix64(np.array([(seed & 0xFFFFFF) * 8 + layer * 2 + which + 0x5151], dtype=_U64))[0]
        fp16_exact = bool(int(pick) % 3 != 0)
    salt = 0
    while True:
        h = splitmix64(np.arange(n, dtype=_U64) ^ (_U64(seed & 0xFFFFFF) << _U64(8)) ^ (_U64(layer * 4 + which) << _U64(32))
                       ^ (_U64(salt) << _U64(48)))
        u = ((h >> _U64(11)).astype(np.float64) / float(1 << 53)) * 2.0 - 1.0
        u = np.sort(u)
        u[0], u[-1] = -1.0, 1.0
        lut = u.astype(np.float16).astype(np.float32)
        if np.all(np.diff(lut) >= 2.0 ** -7):
            return lut if fp16_exact else u.astype(np.float32)
        salt += 1


def calibrate_k(w: Workload, layer: int = 0, n_cal: int = 4096, profile=None):
    """Stand-in for the offline per-channel Key calibration.

    Draws n_cal calibration tokens (their own tensor id, so they never coincide with cached
    tokens), and per channel takes the (p/2) and (1-p/2) order statistics as outlier
    thresholds and the mid-/half-range of the values strictly inside as zero-point / scale.
    Returns float16 arrays s, z, lo, hi of shape [D]."""
    x = gen_k(w, layer, 0, 0, n_cal, profile=profile, tensor_id=T_KCAL).astype(np.float32)
    xs = np.sort(x, axis=0)
    k = int(round(w.outlier_fraction / 2.0 * n_cal))
    if k > 0:
        lo = xs[k - 1, :]
        hi = xs[n_cal - k, :]
        inner_min = xs[k, :]
        inner_max = xs[n_cal - k - 1, :]
    else:
        inner_min = xs[0, :]
        inner_max = xs[-1, :]
        lo = np.full(w.D, -65504.0, dtype=np.float32)
        hi = np.full(w.D, 65504.0, dtype=np.float32)
    z = ((inner_max + inner_min) * np.float32(0.5)).astype(np.float16)
    s = ((inner_max - inner_min) * np.float32(0.5)).astype(np.float16)
    s = np.where(s.astype(np.float32) <= 0, np.float16(1.0), s)
    return s, z, lo.astype(np.float16), hi.astype(np.float16)


T_CALX, T_CALW = 9, 10


def gen_calibration(seed: int, n: int, layer: int = 0):
    """Stand-in for the inputs of the offline datatype derivation: n normalised calibration
    activations in [-1, 1] and their sensitivity weights (Fisher information times squared scale).

    Values: bell-shaped, with a width that depends on the element's channel (i mod 128), clipped to
    [-1, 1]; one element in 257 sits exactly on an end of the range (every normalised vector touches
    both ends).  Weights: log-normal times a per-channel factor, one in 64 exactly zero (elements
    the loss does not depend on).  Both fp32; element i depends on (seed, layer, i) only."""
    i = np.arange(n, dtype=_U64)
    key = _U64(seed) ^ (_U64(layer) << _U64(48))
    hx = splitmix64(key ^ (_U64(T_CALX) << _U64(56)) ^ i)
    hw = splitmix64(key ^ (_U64(T_CALW) << _U64(56)) ^ i)
    ch = (i % _U64(128)).astype(np.int64)
    width = (np.float32(0.18) + np.float32(0.30) * ((ch * 37) % 128).astype(np.float32) / np.float32(128.0))
    x = np.clip(normalish(hx).reshape(-1) * width, -1.0, 1.0).astype(np.float32)
    h2 = splitmix64(hx)
    end = (h2 % _U64(257)) == 0
    x = np.where(end, np.where((h2 >> _U64(20)) & _U64(1), np.float32(1.0), np.float32(-1.0)), x).astype(np.float32)
    g = normalish(hw).reshape(-1)
    chan = (np.float32(0.25) + ((ch * 53) % 128).astype(np.float32) / np.float32(64.0)) ** 2
    w = (np.exp(np.float32(1.5) * g).astype(np.float32) * chan.astype(np.float32)).astype(np.float32)
    w = np.where((splitmix64(hw) % _U64(64)) == 0, np.float32(0.0), w).astype(np.float32)
    return x, w


class LayerInputs:
    """Everything one synthetic attention layer feeds the method with: look-up tables, per-channel Key
    calibration constants, the Value outlier count per side, and the token generators."""

    def __init__(self, wl: Workload, layer=0):
        self.wl = wl
        self.bits = wl.bits
        self.layer = layer
        self.lut_k = make_lut(wl.bits, wl.seed, layer, 0)
        self.lut_v = make_lut(wl.bits, wl.seed, layer, 1)
        self.kprof = key_channel_profile(wl, layer)
        self.vprof = value_channel_profile(wl, layer)
        self.s, self.z, self.lo, self.hi = calibrate_k(wl, layer, profile=self.kprof)
        self.k_side = k_side_from_fraction(wl.outlier_fraction, wl.D)

    def cap_nnz_k(self, cap):
        """Entries to provide for Key outliers in a cache of `cap` tokens (twice the expected count)."""
        return int(max(1024, 2.0 * max(self.wl.outlier_fraction, 1e-4) * self.wl.D * cap))

    def k(self, t0, T, seq=0):
        return gen_k(self.wl, self.layer, seq, t0, T, profile=self.kprof)

    def v(self, t0, T, seq=0):
        return gen_v(self.wl, self.layer, seq, t0, T, profile=self.vprof)
