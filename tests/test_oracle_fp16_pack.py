"""Pins for the oracle's fp16 conversion and packed-code storage format."""
import json
import os

import numpy as np
import pytest

from oracle import kvq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_h2f_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([O.h2f(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_f2h_matches_numpy_rne_including_ties_and_subnormals():
    rng = np.random.default_rng(7)
    xs = [rng.standard_normal(20000).astype(np.float32) * s for s in (1e-7, 1e-4, 1.0, 300.0, 7e4)]
    # exact halfway points between neighbouring fp16 numbers (ties must go to even)
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    a = h.view(np.float16).astype(np.float64)
    b = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((a + b) / 2).astype(np.float32)
    xs += [mid, -mid, np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 5.96e-8, 2.9e-8, 3.1e-8], np.float32)]
    x = np.concatenate(xs)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = np.array([O.f2h(v) for v in x], dtype=np.uint16)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("H", [1, 8])
def test_pack_unpack_roundtrip_and_size(bits, H):
    cap = 256
    rng = np.random.default_rng(bits * 10 + H)
    D = H * 128
    assert O.codes_bytes(bits, H, cap) == cap * D * bits // 8      # exactly b bits per element
    oc_k = np.zeros(O.codes_bytes(bits, H, cap), np.uint8)
    oc_v = np.zeros_like(oc_k)
    codes = rng.integers(0, 1 << bits, size=(cap - 3, D), dtype=np.uint8)
    O._pack_k(oc_k, bits, H, cap, 3, cap - 3, codes)
    O._pack_v(oc_v, bits, H, cap, 3, cap - 3, codes)
    back = np.zeros_like(codes)
    O._unpack_k(oc_k, bits, H, cap, 3, cap - 3, back)
    assert np.array_equal(back, codes)
    back[:] = 0
    O._unpack_v(oc_v, bits, H, cap, 3, cap - 3, back)
    assert np.array_equal(back, codes)
    # the three never-written tokens stay zero, and every bit of the written region is used:
    # all-ones codes fill the written tokens' bytes completely
    ones = np.full((cap, D), (1 << bits) - 1, np.uint8)
    full = np.zeros_like(oc_k)
    O._pack_k(full, bits, H, cap, 0, cap, ones)
    assert np.all(full == 0xFF)
    full[:] = 0
    O._pack_v(full, bits, H, cap, 0, cap, ones)
    assert np.all(full == 0xFF)


def test_pack_overwrite_only_touches_own_bits():
    bits, H, cap = 3, 2, 128
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 8, size=(cap, H * 128), dtype=np.uint8)
    buf = np.zeros(O.codes_bytes(bits, H, cap), np.uint8)
    O._pack_v(buf, bits, H, cap, 0, cap, codes)
    new = rng.integers(0, 8, size=(1, H * 128), dtype=np.uint8)
    O._pack_v(buf, bits, H, cap, 77, 1, new)          # odd token shares fields with token 76
    codes[77] = new[0]
    back = np.zeros_like(codes)
    O._unpack_v(buf, bits, H, cap, 0, cap, back)
    assert np.array_equal(back, codes)


def test_hand_derived_byte_images():
    with open(os.path.join(GOLDEN, "pack_examples.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        bits, H, cap = case["bits"], case["n_kv_heads"], case["cap"]
        buf = np.zeros(O.codes_bytes(bits, H, cap), np.uint8)
        put = O._lib.kvqo_k_put if case["kind"] == "k" else O._lib.kvqo_v_put
        for n, ch, code in case["writes"]:
            put(buf.ctypes.data_as(O.C.c_void_p), bits, O.C.c_int64(cap), O.C.c_int64(n), ch, code)
        expect = np.zeros_like(buf)
        for off, val in case["nonzero"].items():
            expect[int(off)] = val
        bad = np.nonzero(buf != expect)[0]
        assert bad.size == 0, (case["name"], bad[:8], buf[bad[:8]], expect[bad[:8]])
