"""Device-side generation of the synthetic Key / Value activations (same values as gen.py)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

from . import gen

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gen_hip.hip")
LIB = os.path.join(HERE, "libkvq_synth.so")
_lib = None


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-o", LIB, SRC]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(r.stdout)
    return LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise ImportError(f"{LIB} is missing: build it first (kvq_synth.device.build())")
        _lib = C.CDLL(LIB)
        _lib.kvq_synth_fill.restype = C.c_int
        _lib.kvq_synth_fill.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def _key(seed, tensor_id, layer, seq) -> int:
    return (int(seed) ^ (tensor_id << 56) ^ (layer << 48) ^ (seq << 40)) & 0xFFFFFFFFFFFFFFFF


class DeviceGen:
    """Holds the per-channel profiles on the device and fills fp16 [T][D] tensors."""

    def __init__(self, w: gen.Workload, layer: int = 0, kprof=None, vprof=None, device="cuda:0"):
        self.w, self.layer = w, layer
        ka, kmu = kprof if kprof is not None else gen.key_channel_profile(w, layer)
        va, vmu = vprof if vprof is not None else gen.value_channel_profile(w, layer)
        dev = torch.device(device)
        self.ka, self.kmu = torch.from_numpy(ka).to(dev), torch.from_numpy(kmu).to(dev)
        self.va, self.vmu = torch.from_numpy(va).to(dev), torch.from_numpy(vmu).to(dev)
        self.dev = dev

    def _fill(self, tensor_id, seq, t0, T, a, mu, row_scale, out):
        if out is None:
            out = torch.empty((T, self.w.D), dtype=torch.float16, device=self.dev)
        assert out.is_contiguous() and out.shape == (T, self.w.D) and out.dtype == torch.float16
        st = _load().kvq_synth_fill(_key(self.w.seed, tensor_id, self.layer, seq), t0, T, self.w.D, a.data_ptr(),
                                    mu.data_ptr(), row_scale.data_ptr() if row_scale is not None else None,
                                    out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if st != 0:
            raise RuntimeError(f"kvq_synth_fill failed ({st})")
        return out

    def k(self, t0, T, seq=0, out=None):
        return self._fill(gen.T_K, seq, t0, T, self.ka, self.kmu, None, out)

    def v(self, t0, T, seq=0, out=None):
        sig = torch.from_numpy(gen.value_token_scale(self.w, self.layer, seq, t0, T)).to(self.dev)
        return self._fill(gen.T_V, seq, t0, T, self.va, self.vmu, sig, out)
