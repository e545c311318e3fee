"""Seeded synthetic inputs for the quantized-KV decode path.

This package only produces INPUTS (activations, queries, look-up tables, per-channel
calibration constants, normalised calibration samples with sensitivity weights).  It contains none of the arithmetic of the method under test
(no quantisation, packing, rotation or mat-vec), so the CPU oracle and the GPU library
can both be fed from it without sharing any code with each other.
"""
from .gen import (  # noqa: F401
    SEED_BASE, Workload, WORKLOADS, workload, splitmix64, hash_grid, normalish,
    key_channel_profile, value_channel_profile, value_token_scale,
    gen_k, gen_v, gen_q, gen_probs_logits, make_lut, calibrate_k, k_side_from_fraction, LayerInputs,
    gen_calibration,
)
