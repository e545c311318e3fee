"""Benchmark of the quantized-KV decode hot path on one MI355X.

A step is one pass of the whole path over the cached context: quantize-append the new token's Key
and Value, q.K^T against the quantized Keys (RoPE after de-quantisation, sparse outliers merged),
softmax, p.V against the quantized Values.  Workload: LLaMA-7B attention layer shape (32 heads x 128),
context 131072, batch 1, 3-bit NUQ with 1 % outliers, seeded synthetic activations.
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

# Kernel arguments in device memory: by default the HIP runtime keeps the argument blocks of launches in
# host memory, and every kernel's first scalar load then crosses the host link (measured here: 1.2 us per
# kernel, 6 us of a 161 us decode step).  HIP_FORCE_DEV_KERNARG is the runtime's own switch for it (AMD's
# tuning guides recommend it on MI300-class GPUs); it must be set before the runtime starts, which is why
# it is set here and not in the library.  --host-kernarg (or the variable set to 0 by the caller) keeps
# the default.  The line reports which one it ran with.
if "--host-kernarg" not in sys.argv:
    os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def build_cache(st, L, cap, K, torch, keep_fp16=False):
    """Fill a GPU cache with L synthetic tokens generated on the device, in chunks of 4096."""
    from kvq_synth.device import DeviceGen
    dg = DeviceGen(st.wl, st.layer, st.kprof, st.vprof)
    wl = st.wl
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap))
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    k16 = torch.empty((L, st.wl.D), dtype=torch.float16, device="cuda") if keep_fp16 else None
    v16 = torch.empty((L, st.wl.D), dtype=torch.float16, device="cuda") if keep_fp16 else None
    t0 = 0
    while t0 < L:
        T = min(4096, L - t0)
        k = dg.k(t0, T, out=k16[t0:t0 + T] if keep_fp16 else None)
        v = dg.v(t0, T, out=v16[t0:t0 + T] if keep_fp16 else None)
        K.kvq_quantize_append_k(gc, k)
        K.kvq_quantize_append_v(gc, v)
        t0 += T
    torch.cuda.synchronize()
    return gc, dg, k16, v16


def bulk_append_rate(st, dg, K, torch, T=4096, calls=4):
    """Prefill-style compression: `calls` appends of T tokens each (Keys and Values) into a small cache
    of its own, inputs resident in HBM; returns the best call's tokens/s and input GB/s."""
    wl = st.wl
    cap = (calls + 1) * T
    gc = K.KvqCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.cap_nnz_k(cap))
    K.kvq_lut_load(gc, st.lut_k, st.lut_v, st.s, st.z, st.lo, st.hi)
    ks = [dg.k(i * T, T) for i in range(calls + 1)]
    vs = [dg.v(i * T, T) for i in range(calls + 1)]
    K.kvq_quantize_append_kv(gc, ks[0], vs[0])             # warm-up
    tm = K.HipEventTimer()
    best = None
    for i in range(1, calls + 1):
        tm.start()
        K.kvq_quantize_append_kv(gc, ks[i], vs[i])
        tm.stop()
        us = tm.elapsed_ms() * 1e3
        best = us if best is None else min(best, us)
    assert gc.status() == 0
    return {"tokens_per_call": T, "us_per_call": best, "tokens_per_s": T / (best * 1e-6),
            "input_gbps": 2 * T * wl.D * 2 / (best * 1e-6) / 1e9}


def calibration_rate(bits, K, torch, n=1 << 26, iters=10):
    """Offline datatype derivation (weighted k-means over n normalised values and weights resident in
    HBM): time per iteration and the rate at which an iteration streams its 8 bytes per element."""
    x = torch.empty(n, device="cuda").normal_(0, 0.3).clamp_(-1, 1)
    w = torch.empty(n, device="cuda").log_normal_(0, 1.5)
    c0 = np.linspace(-1, 1, 1 << bits).astype(np.float32)
    K.kvq_calibrate_nuq(x, w, bits, 1, c0)                 # warm-up
    torch.cuda.synchronize()
    t = time.perf_counter()
    K.kvq_calibrate_nuq(x, w, bits, iters, c0)             # synchronizes before it returns
    dt = (time.perf_counter() - t) / iters
    return {"elements": n, "bits": bits, "us_per_iteration": dt * 1e6, "gbps": 8 * n / dt / 1e9}


KERNEL_SOURCES = ("kvq_qk.hip", "kvq_qk_sparse.hpp", "kvq_pv.hip", "kvq_common.hpp")


def kernel_source_hash():
    """SHA-256 over the sources of the attention kernels, as the counter summaries under profiles/ name it."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2401_18079_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def profile_constants(fname, keys):
    """`key: value` lines of a counter summary under profiles/, or None when the file is missing, lacks a
    key, or was taken with other kernel sources than the tree holds."""
    path = os.path.join(ROOT, "profiles", fname)
    if not os.path.exists(path):
        return None
    kv = {}
    for ln in open(path):
        if ":" in ln:
            k, v = ln.split(":", 1)
            kv[k.strip()] = v.strip()
    if kv.get("kernel_source_sha256") != kernel_source_hash():
        return None
    try:
        return {k: float(kv[k]) for k in keys}
    except (KeyError, ValueError):
        return None


def algorithmic_bytes(wl, L, nnz_k, nnz_v):
    """Bytes the method must move per launch (compressed cache + outputs), not the fp16 bytes it avoids."""
    D, Hq, b = wl.D, wl.n_q_heads, wl.bits
    qk = L * (D * b // 8) + 4 * nnz_k + 4 * (L + 1) + 4 * Hq * L
    pv = L * (D * b // 8) + 4 * L + 4 * nnz_v + 4 * (L + 1) + 4 * Hq * L
    return qk, pv


def cpu_baseline(st, sample_tokens):
    """Time the CPU oracle (as it stands) on a bounded sample of the same workload."""
    import kvq_synth as S
    from oracle import kvq_oracle as O
    wl = st.wl
    cap = ((sample_tokens + 127) // 128) * 128
    oc = O.OracleCache(wl.bits, wl.n_kv_heads, wl.n_q_heads, cap, st.k_side, wl.rope_base, st.lut_k, st.lut_v,
                       st.s, st.z, st.lo, st.hi, cap_nnz_k=st.cap_nnz_k(cap))
    t0 = 0
    tq = 0.0
    while t0 < sample_tokens:                       # cache construction is not timed, except one token
        T = min(1024, sample_tokens - t0)
        k, v = st.k(t0, T), st.v(t0, T)
        if t0 + T == sample_tokens:
            oc.append_k(k[:-1]); oc.append_v(v[:-1])
            a = time.perf_counter()
            oc.append_k(k[-1:]); oc.append_v(v[-1:])
            tq = time.perf_counter() - a
        else:
            oc.append_k(k); oc.append_v(v)
        t0 += T
    q = S.gen_q(wl, 0, 0)
    times = []
    for _ in range(5):
        a = time.perf_counter()
        scores = oc.qk(q, 1.0 / np.sqrt(128.0))
        probs = O.softmax(scores)
        out = oc.pv(probs)
        times.append(time.perf_counter() - a)
    return tq, float(np.median(times)), O.max_threads(), float(out[0, 0])


def model_step(args, wl, S, K, torch):
    """`--layers N`: one decode step of N attention layers, each with its own cache, look-up tables and
    per-channel constants (the full-model configuration: 32 layers at a context of 2^20 tokens keep
    ~110 GB of compressed cache resident).  Per layer: kvq_decode_step."""
    L, steps, warmup, n_layers = wl.context, args.steps, args.warmup, args.layers
    n_new = steps + warmup
    cap = ((L + n_new + 8 + 127) // 128) * 128
    Hq = wl.n_q_heads
    scale = 1.0 / np.sqrt(128.0)
    caches, new_k, new_v = [], [], []
    t0 = time.perf_counter()
    for layer in range(n_layers):
        st = S.LayerInputs(wl, layer)
        gc, dg, _, _ = build_cache(st, L, cap, K, torch)
        assert gc.status() == 0
        caches.append(gc)
        new_k.append(dg.k(L, n_new))
        new_v.append(dg.v(L, n_new))
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    qs = torch.from_numpy(np.stack([S.gen_q(wl, 0, 0, step=i) for i in range(n_new)])).cuda()
    scores = torch.zeros((Hq, cap), device="cuda")           # scratch shared by the layers
    out = torch.zeros((n_layers, Hq, 128), device="cuda")

    def step(i):
        for layer, gc in enumerate(caches):
            K.kvq_decode_step(gc, new_k[layer][i:i + 1], new_v[layer][i:i + 1], qs[i], scale, scores, out[layer])

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t_begin) * 1e3 / steps
    for gc in caches:
        assert gc.status() == 0
    tensors = ("params", "k_codes", "v_codes", "v_sz", "k_ptr", "v_ptr", "k_idx", "k_val", "v_idx", "v_val", "workspace")
    resident = sum(getattr(gc, t).numel() * getattr(gc, t).element_size() for gc in caches for t in tensors)
    gc = caches[0]
    Lend = gc.n_tokens_k
    nnz_k = int(gc.k_ptr[Lend].item()) & 0xFFFFFFFF
    nnz_v = int(gc.v_ptr[Lend].item()) & 0xFFFFFFFF
    qk_bytes, pv_bytes = algorithmic_bytes(wl, Lend, nnz_k, nnz_v)
    line = {
        "metric": "quantized-KV decode step latency over all layers (per layer: append K/V + QK^T + softmax + PV)",
        "value": ms, "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {n_layers} layers x {wl.n_q_heads} q-heads x {wl.n_kv_heads} kv-heads x 128, "
                               f"context {L}, batch 1, nuq{wl.bits} with {wl.outlier_fraction * 100:g}% outliers",
                   "layers": n_layers, "bits": wl.bits, "context": L, "outlier_fraction": wl.outlier_fraction},
        "us_per_layer": ms * 1e3 / n_layers,
        "resident_cache_gb": resident / 1e9,
        "cache_build_s": build_s,
        "hbm_gbps_algorithmic": n_layers * (qk_bytes + pv_bytes) / (ms * 1e-3) / 1e9,
    }
    print(json.dumps(line))

def million_token_leg(args, K, S, torch):
    """Configuration 3 beside the headline workload: the same layer shape at a context of 1,048,576 tokens,
    nuq4 with 0.1 % outliers, where a step first quantize-appends 64 new tokens (Keys and Values) and then
    runs the attention (scores, softmax, output) over the whole context.  Returns the dictionary that
    the bench line carries under "c3"."""
    wl = S.workload("c3")
    st = S.LayerInputs(wl)
    L, T = wl.context, 64
    steps = max(4, min(args.steps, 40))
    warmup = max(2, min(args.warmup, 5))
    bsteps = max(4, min(steps, 20))
    n_calls = warmup + steps + 3 * bsteps
    cap = ((L + n_calls * T + 8 + 127) // 128) * 128
    Hq, D = wl.n_q_heads, wl.D
    scale = 1.0 / np.sqrt(128.0)
    gc, dg, k16, v16 = build_cache(st, L, cap, K, torch, keep_fp16=not args.no_fp16)
    assert gc.status() == 0
    new_k = dg.k(L, n_calls * T)
    new_v = dg.v(L, n_calls * T)
    q = torch.from_numpy(S.gen_q(wl, 0, 0)).cuda()
    scores = torch.zeros((Hq, cap), device="cuda")
    out = torch.zeros((Hq, 128), device="cuda")

    def step(i, ev=None):
        K.kvq_quantize_append_kv(gc, new_k[i * T:(i + 1) * T], new_v[i * T:(i + 1) * T])
        if ev: ev[1].start()  # noqa: E701
        K.kvq_attention_decode(gc, q, scale, scores, out)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    us_per_step = (time.perf_counter() - t_begin) * 1e6 / steps
    base = warmup + steps
    evs = [[K.HipEventTimer() for _ in range(3)] for _ in range(bsteps)]
    for i in range(bsteps):
        evs[i][0].start()
        step(base + i, evs[i])
        evs[i][2].start()
    torch.cuda.synchronize()
    import ctypes
    lib = K.load_library()

    def gap_us(a, b):
        ms = ctypes.c_float()
        lib.kvq_event_elapsed_ms(a._a, b._a, ctypes.byref(ms))
        return ms.value * 1e3

    append_us = float(np.mean([gap_us(e[0], e[1]) for e in evs]))
    attention_us = float(np.mean([gap_us(e[1], e[2]) for e in evs]))
    base += bsteps
    # the dense kernels inside back-to-back steps: the Value kernel by its workgroups' span, the Key
    # kernel (eight query heads per thread: no span-taking variant) by the HIP-event interval around
    # its launch, which is an upper bound on its duration
    K.kvq_profile_enable(True, spans=True, events=False)
    for i in range(bsteps):
        step(base + i)
    torch.cuda.synchronize()
    K.kvq_profile_enable(False)
    dense_pv = K.kvq_profile_read_all_spans_us(1)
    try:
        dense_qk = K.kvq_profile_read_all_spans_us(0)
        qk_how = "span of the kernel's workgroups on the GPU wall clock"
    except K.KvqError:
        dense_qk = None
    K.kvq_profile_enable(True)
    for i in range(bsteps):
        step(base + bsteps + i)
    torch.cuda.synchronize()
    K.kvq_profile_enable(False)
    ev_qk = K.kvq_profile_read_all_us(0)
    if dense_qk is None:
        dense_qk = ev_qk
        qk_how = "interval between HIP events recorded around the launch (an upper bound: no span-taking variant of this kernel)"
    Lend = gc.n_tokens_k
    assert gc.status() == 0 and Lend == L + n_calls * T
    nnz_k = int(gc.k_ptr[Lend].item()) & 0xFFFFFFFF
    nnz_v = int(gc.v_ptr[Lend].item()) & 0xFFFFFFFF
    qk_bytes, pv_bytes = algorithmic_bytes(wl, Lend, nnz_k, nnz_v)
    append_bytes = T * (2 * (2 * D) + 2 * (D * wl.bits // 8) + 12) + 4 * (nnz_k + nnz_v) * T // Lend
    dense_qk_us = float(np.mean(dense_qk))
    dense_qk_bytes = Lend * (D * wl.bits // 8) + 4 * Hq * Lend
    dense_qk_gbps = dense_qk_bytes / (dense_qk_us * 1e-6) / 1e9
    fp16 = None
    if not args.no_fp16:
        probs = torch.softmax(scores[:, :L], dim=1).contiguous()
        s16 = torch.zeros((Hq, L), device="cuda")
        fws = torch.zeros(K.binding.kvq_fp16_pv_workspace_bytes(Hq, L), dtype=torch.uint8, device="cuda")
        tm = K.HipEventTimer()
        res = {}
        for name, fn in (("qk", lambda: K.kvq_fp16_qk_matvec(k16, wl.n_kv_heads, Hq, q, scale, s16)),
                         ("pv", lambda: K.kvq_fp16_pv_matvec(v16, wl.n_kv_heads, Hq, probs, out, fws))):
            for _ in range(2):
                fn()
            tm.start()
            for _ in range(5):
                fn()
            tm.stop()
            res[name] = tm.elapsed_ms() * 1e3 / 5
        fp16 = {"qk_us": res["qk"], "pv_us": res["pv"], "qk_gbps": L * D * 2 / (res["qk"] * 1e-6) / 1e9,
                "pv_gbps": L * D * 2 / (res["pv"] * 1e-6) / 1e9}
        del k16, v16, probs, s16, fws
    total_bytes = qk_bytes + pv_bytes + append_bytes
    return {
        "config": {"workload": f"c3: {Hq} q-heads x {wl.n_kv_heads} kv-heads x 128, context {L}, batch 1, "
                               f"nuq{wl.bits} with {wl.outlier_fraction * 100:g}% outliers, a step appends {T} new tokens "
                               f"(Keys and Values) before the mat-vecs",
                   "bits": wl.bits, "context": L, "outlier_fraction": wl.outlier_fraction, "append_tokens": T},
        "step": "kvq_quantize_append_kv (64 tokens) + kvq_attention_decode",
        "value": us_per_step, "unit": "us", "steps": steps, "warmup": warmup,
        "breakdown_us": {"append_kv_64_tokens": append_us, "attention_decode": attention_us},
        "algorithmic_bytes": {"qk": qk_bytes, "pv": pv_bytes, "append": append_bytes},
        "hbm_gbps_step": total_bytes / (us_per_step * 1e-6) / 1e9,
        "hbm_gbps_attention": (qk_bytes + pv_bytes) / (attention_us * 1e-6) / 1e9,
        "dense_kernel_us": {"qk": dense_qk_us, "qk_measured": qk_how, "pv": float(np.mean(dense_pv)),
                            "pv_measured": "span of the kernel's workgroups on the GPU wall clock",
                            "qk_event_interval_us": float(np.mean(ev_qk)), "launches": bsteps},
        "roofline": {"bound": "hbm", "kernel": "kvq_qk_kernel<4 bits> (dense Key kernel of the attention call)",
                     "achieved": dense_qk_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": dense_qk_gbps / HBM_PEAK_GBPS,
                     "traffic": (profile_constants("kvq_qk_kernel_c3_hbm_traffic.txt",
                                                   ("dense_kernel_traffic_bytes_per_launch",))
                                 or {}).get("dense_kernel_traffic_bytes_per_launch"),
                     "algorithmic_bytes": dense_qk_bytes, "avg_launch_us": dense_qk_us},
        "fp16_cache_baseline": fp16,
        "speedup_vs_fp16_attention": ((fp16["qk_us"] + fp16["pv_us"]) / attention_us) if fp16 else None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--context", type=int, default=0, help="override the context length")
    ap.add_argument("--bits", type=int, default=0, help="override the code width (2, 3 or 4)")
    ap.add_argument("--outliers", type=float, default=-1.0, help="override the outlier fraction (e.g. 0.01)")
    ap.add_argument("--cpu-sample", type=int, default=16384, help="tokens of context for the CPU-oracle timing (0 = skip)")
    ap.add_argument("--layers", type=int, default=1,
                    help="more than 1: time a decode step over that many layers (each its own cache), nothing else")
    ap.add_argument("--no-fp16", action="store_true")
    ap.add_argument("--no-c3", action="store_true", help="skip the 1M-token leg (configuration 3) of the default run")
    ap.add_argument("--host-kernarg", action="store_true",
                    help="leave kernel arguments in host memory (the HIP runtime's default) instead of setting "
                         "HIP_FORCE_DEV_KERNARG=1")
    ap.add_argument("--print-source-hash", action="store_true",
                    help="print the hash of the attention kernels' sources (the one a counter summary must name) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device copy (known traffic) so profiler byte counters can be scaled")
    args = ap.parse_args()
    if args.print_source_hash:
        print(kernel_source_hash())
        return
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import kvq_synth as S
    import paper_2401_18079_amd as K

    over = {}
    if args.context:
        over["context"] = args.context
    if args.bits:
        over["bits"] = args.bits
    if args.outliers >= 0:
        over["outlier_fraction"] = args.outliers
    wl = S.workload(args.workload, **over)
    if args.layers > 1:
        model_step(args, wl, S, K, torch)
        return
    st = S.LayerInputs(wl)
    L = wl.context
    steps, warmup = args.steps, args.warmup
    bsteps = min(steps, 200)                       # extra steps timed call by call for the breakdowns
    steps3 = min(steps, 200)                       # extra steps made of five separate calls
    n_new = steps + warmup + 4 * bsteps + steps3 + 5
    cap = ((L + n_new + 8 + 127) // 128) * 128
    Hq, D = wl.n_q_heads, wl.D
    scale = 1.0 / np.sqrt(128.0)

    gc, dg, k16, v16 = build_cache(st, L, cap, K, torch, keep_fp16=not args.no_fp16)
    assert gc.status() == 0
    new_k = dg.k(L, n_new)
    new_v = dg.v(L, n_new)
    qs = torch.from_numpy(np.stack([S.gen_q(wl, 0, 0, step=i) for i in range(n_new)])).cuda()
    scores = torch.zeros((Hq, cap), device="cuda")
    probs = torch.zeros((Hq, cap), device="cuda")
    out = torch.zeros((Hq, 128), device="cuda")
    sm_ws = torch.zeros(K.binding.kvq_softmax_workspace_bytes(Hq, cap), dtype=torch.uint8, device="cuda")

    def step(i, ev=None, fused=True):
        """One decode step of one attention layer.  fused: one library call (kvq_decode_step: the appends
        of Keys and Values in one launch, then scores, softmax and output with the softmax folded into
        the mat-vec kernels), or its two halves as two calls when an event goes between them;
        otherwise the same work as five separate calls."""
        if fused and ev is None:
            K.kvq_decode_step(gc, new_k[i:i + 1], new_v[i:i + 1], qs[i], scale, scores, out)   # both halves in one call
            return
        if fused:
            K.kvq_quantize_append_kv(gc, new_k[i:i + 1], new_v[i:i + 1])
            ev[1].start()
            K.kvq_attention_decode(gc, qs[i], scale, scores, out)
            return
        K.kvq_quantize_append_k(gc, new_k[i:i + 1])
        if ev: ev[1].start()  # noqa: E701
        K.kvq_quantize_append_v(gc, new_v[i:i + 1])
        if ev: ev[2].start()  # noqa: E701
        K.kvq_qk_matvec(gc, qs[i], scale, scores)
        if ev: ev[3].start()  # noqa: E701
        K.kvq_softmax_f32(scores, probs, gc.n_tokens_k, sm_ws)
        if ev: ev[4].start()  # noqa: E701
        K.kvq_pv_matvec(gc, probs, out)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # the timed region: exactly `steps` steps, nothing else on the stream
    t_begin = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    ms_per_step = wall * 1e3 / steps

    # the same steps as five separate calls (append k, append v, qk, softmax, pv)
    base = warmup + steps
    for i in range(5):
        step(base + i, fused=False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(steps3):
        step(base + 5 + i, fused=False)
    torch.cuda.synchronize()
    ms_per_step_separate = (time.perf_counter() - t_begin) * 1e3 / steps3
    base += 5 + steps3

    # per-call breakdowns from further steps, with an event recorded on the launch stream between the
    # calls (start() records one event); the events themselves cost a few microseconds per step, which
    # is why they stay out of the timed regions above
    evs = [[K.HipEventTimer() for _ in range(6)] for _ in range(bsteps)]
    for i in range(bsteps):
        ev = evs[i]
        ev[0].start()
        step(base + i, ev, fused=False)
        ev[5].start()
    fevs = [[K.HipEventTimer() for _ in range(3)] for _ in range(bsteps)]
    for i in range(bsteps):
        ev = fevs[i]
        ev[0].start()
        step(base + bsteps + i, ev, fused=True)
        ev[2].start()
    torch.cuda.synchronize()

    import ctypes
    lib = K.load_library()

    def gap_ms(a, b):
        ms = ctypes.c_float()
        lib.kvq_event_elapsed_ms(a._a, b._a, ctypes.byref(ms))
        return ms.value

    names = ["append_k", "append_v", "qk_matvec", "softmax", "pv_matvec"]
    per = {n: [] for n in names}
    for ev in evs:
        for j, n in enumerate(names):
            per[n].append(gap_ms(ev[j], ev[j + 1]) * 1e3)
    breakdown = {n: float(np.mean(v)) for n, v in per.items()}
    breakdown_min = {n: float(np.min(v)) for n, v in per.items()}
    breakdown_median = {n: float(np.median(v)) for n, v in per.items()}
    fnames = ["append_kv", "attention_decode"]
    fper = {n: [gap_ms(ev[j], ev[j + 1]) * 1e3 for ev in fevs] for j, n in enumerate(fnames)}
    fused_breakdown = {n: float(np.mean(v)) for n, v in fper.items()}
    fused_breakdown_stats = {n: {"median": float(np.median(v)), "min": float(np.min(v)), "samples": len(v)}
                             for n, v in fper.items()}

    Lend = gc.n_tokens_k
    nnz_k = int(gc.k_ptr[Lend].item()) & 0xFFFFFFFF
    nnz_v = int(gc.v_ptr[Lend].item()) & 0xFFFFFFFF
    qk_bytes, pv_bytes = algorithmic_bytes(wl, Lend, nnz_k, nnz_v)
    qk_gbps = qk_bytes / (breakdown["qk_matvec"] * 1e-6) / 1e9
    pv_gbps = pv_bytes / (breakdown["pv_matvec"] * 1e-6) / 1e9

    # the dominant kernel on its own, inside full decode steps run back to back exactly like the timed
    # region (same workload, same launch configuration, no wait for the GPU between steps).  Its
    # duration is the kernel's own span (first wavefront start to last wavefront end on the GPU's wall
    # clock, which is what a kernel trace reports); the interval between HIP events recorded around the
    # launch is taken in further steps and reported beside it: the event records stall the queue, so
    # that interval is an upper bound (by 1 to 7 us, depending on the machine)
    base = warmup + steps + 5 + steps3 + 2 * bsteps
    K.kvq_profile_enable(True, spans=True, events=False)
    for i in range(bsteps):
        step(base + i)
    torch.cuda.synchronize()
    K.kvq_profile_enable(False)
    measured = ("span of the kernel's workgroups on the GPU wall clock, %d launches inside back-to-back "
                "decode steps" % bsteps)
    dense_pv = K.kvq_profile_read_all_spans_us(1)
    try:
        dense_qk = K.kvq_profile_read_all_spans_us(0)
    except K.KvqError:
        dense_qk = None                     # no span-taking variant of this shape's kernel (eight heads per thread)
    K.kvq_profile_enable(True)
    for i in range(bsteps):
        step(base + bsteps + i)
    torch.cuda.synchronize()
    K.kvq_profile_enable(False)
    ev_qk, ev_pv = K.kvq_profile_read_all_us(0), K.kvq_profile_read_all_us(1)
    if dense_qk is None:
        dense_qk = ev_qk
        measured = ("qk: interval between HIP events recorded around the launch (upper bound); pv: span of the "
                    "kernel's workgroups on the GPU wall clock; %d launches inside back-to-back decode steps" % bsteps)
    assert len(dense_qk) == bsteps and len(dense_pv) == bsteps
    dense_qk_us, dense_pv_us = float(np.mean(dense_qk)), float(np.mean(dense_pv))
    # dense kernel: packed codes in, fp32 scores out (the sparse kernel's bytes are counted with the call)
    dense_qk_bytes = Lend * (D * wl.bits // 8) + 4 * Hq * Lend
    dense_qk_gbps = dense_qk_bytes / (dense_qk_us * 1e-6) / 1e9

    fp16 = None
    if not args.no_fp16:
        fws = torch.zeros(K.binding.kvq_fp16_pv_workspace_bytes(Hq, L), dtype=torch.uint8, device="cuda")
        K.kvq_softmax_f32(scores, probs, gc.n_tokens_k, sm_ws)
        p16 = probs[:, :L].contiguous()
        s16 = torch.zeros((Hq, L), device="cuda")
        tm = K.HipEventTimer()
        res = {}
        for name, fn in (("qk", lambda: K.kvq_fp16_qk_matvec(k16, wl.n_kv_heads, Hq, qs[0], scale, s16)),
                         ("pv", lambda: K.kvq_fp16_pv_matvec(v16, wl.n_kv_heads, Hq, p16, out, fws))):
            for _ in range(5):
                fn()
            tm.start()
            for _ in range(20):
                fn()
            tm.stop()
            res[name] = tm.elapsed_ms() * 1e3 / 20
        # library cross-check of the same fp16 mat-vecs
        kk = k16.view(L, wl.n_kv_heads, 128)
        qv = qs[0].view(wl.n_kv_heads, Hq // wl.n_kv_heads, 128)
        for _ in range(3):
            torch.einsum("lhc,hrc->hrl", kk.float() if False else kk, qv.half())
        tm.start()
        for _ in range(10):
            torch.einsum("lhc,hrc->hrl", kk, qv.half())
        tm.stop()
        res["qk_torch"] = tm.elapsed_ms() * 1e3 / 10
        fp16 = {"qk_us": res["qk"], "pv_us": res["pv"], "qk_torch_einsum_us": res["qk_torch"],
                "qk_gbps": L * D * 2 / (res["qk"] * 1e-6) / 1e9, "pv_gbps": L * D * 2 / (res["pv"] * 1e-6) / 1e9}
        del k16, v16

    # what a kernel that only reads reaches on this GPU (4 GiB: sixteen times the last-level cache)
    sbuf = torch.ones(1 << 32, dtype=torch.uint8, device="cuda")
    sws = torch.zeros(K.binding.kvq_stream_read_workspace_bytes(), dtype=torch.uint8, device="cuda")
    tm = K.HipEventTimer()
    for _ in range(3):
        K.binding.kvq_stream_read(sbuf, sws)
    tm.start()
    for _ in range(10):
        K.binding.kvq_stream_read(sbuf, sws)
    tm.stop()
    stream_gbps = sbuf.numel() / (tm.elapsed_ms() * 1e-3 / 10) / 1e9
    stream_read = {"gbps": stream_gbps, "bytes": sbuf.numel(), "frac_of_peak": stream_gbps / HBM_PEAK_GBPS,
                   "dense_qk_frac_of_stream_read": dense_qk_gbps / stream_gbps}
    del sbuf, sws

    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    bulk = bulk_append_rate(st, dg, K, torch)
    calib = calibration_rate(wl.bits, K, torch)

    cpu = None
    if args.cpu_sample > 0:
        tq, tmv, cores, _ = cpu_baseline(st, args.cpu_sample)
        # the oracle's cost is linear in the context: scale the sample to the benchmark's context
        est_us = (tq + tmv * (L / args.cpu_sample)) * 1e6
        cpu = {"value": est_us, "unit": "us per decode step (append + qk + softmax + pv)", "cores": cores,
               "kind": "oracle",
               "sample": f"oracle timed on the first {args.cpu_sample} tokens of the same workload "
                         f"(append of one token {tq * 1e3:.2f} ms, qk+softmax+pv {tmv * 1e3:.1f} ms, median of 5), "
                         f"mat-vec time scaled linearly to context {L}"}

    # HBM bytes and VALU instructions per launch of the dense Key kernel come from rocprofv3 counter runs of
    # this command (they cannot be read from inside the run), kept as text summaries under profiles/.  A
    # summary names the hash of the kernel sources it was taken with; it is used only while that hash is
    # the hash of the sources in the tree, so a changed kernel reports null instead of a stale figure.
    traffic = profile_constants(f"kvq_qk_kernel_{wl.name}_hbm_traffic.txt", ("dense_kernel_traffic_bytes_per_launch",))
    traffic = traffic["dense_kernel_traffic_bytes_per_launch"] if traffic and not over else None
    valu = None
    kv = profile_constants(f"bench_{wl.name}_valu_issue.txt", ("qk_valu_instructions_per_launch", "valu_issue_peak_per_s"))
    if kv and not over:
        ach = kv["qk_valu_instructions_per_launch"] / (dense_qk_us * 1e-6)
        valu = {"instructions_per_launch": kv["qk_valu_instructions_per_launch"], "achieved": ach,
                "peak": kv["valu_issue_peak_per_s"], "unit": "wavefront VALU instructions/s",
                "frac": ach / kv["valu_issue_peak_per_s"]}

    line = {
        "metric": "quantized-KV decode step latency (append K/V + QK^T + softmax + PV), one attention layer",
        "step": "kvq_decode_step (append of the new token and attention over the cache that ends with it)",
        "step_launches": K.kvq_decode_step_launches(gc),
        "env": {"HIP_FORCE_DEV_KERNARG": os.environ.get("HIP_FORCE_DEV_KERNARG", "")},
        "value": ms_per_step * 1e3, "unit": "us", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_q_heads} q-heads x {wl.n_kv_heads} kv-heads x 128, context {L}, "
                               f"batch 1, nuq{wl.bits} with {wl.outlier_fraction * 100:g}% outliers, "
                               f"rope base {wl.rope_base:g}",
                   "bits": wl.bits, "context": L, "outlier_fraction": wl.outlier_fraction},
        "separate_calls": {"step": "kvq_quantize_append_k + kvq_quantize_append_v + kvq_qk_matvec + kvq_softmax_f32 "
                                   "+ kvq_pv_matvec",
                           "ms_per_step": ms_per_step_separate, "steps": steps3},
        "fused_breakdown_us": fused_breakdown,
        "fused_breakdown_stats_us": fused_breakdown_stats,
        "breakdown_us": breakdown, "breakdown_min_us": breakdown_min, "breakdown_median_us": breakdown_median,
        "qk_pv_us": breakdown["qk_matvec"] + breakdown["pv_matvec"],
        "hbm_gbps": {"qk_matvec": qk_gbps, "pv_matvec": pv_gbps},
        "bulk_append": bulk,
        "calibration": calib,
        "fp16_cache_baseline": fp16,
        "speedup_vs_fp16": ({"qk": fp16["qk_us"] / breakdown["qk_matvec"], "pv": fp16["pv_us"] / breakdown["pv_matvec"]}
                            if fp16 else None),
        "dense_kernel_us": {"qk": dense_qk_us, "pv": dense_pv_us,
                            "qk_median": float(np.median(dense_qk)), "qk_min": float(np.min(dense_qk)),
                            "pv_median": float(np.median(dense_pv)), "pv_min": float(np.min(dense_pv)),
                            "measured": measured,
                            "event_interval_us": {"qk": float(np.mean(ev_qk)), "pv": float(np.mean(ev_pv))}},
        "roofline": {"bound": "hbm", "kernel": "kvq_qk_kernel (dense Key kernel of the attention call)",
                     "achieved": dense_qk_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": dense_qk_gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "algorithmic_bytes": dense_qk_bytes, "avg_launch_us": dense_qk_us,
                     "whole_call": {"algorithmic_bytes": qk_bytes, "avg_us": breakdown["qk_matvec"],
                                    "achieved": qk_gbps, "frac": qk_gbps / HBM_PEAK_GBPS},
                     "stream_read": stream_read,
                     "valu_issue": valu},
        "cpu_baseline": cpu,
    }
    # the 1M-token half of the metric: configuration 3 timed after the headline workload (whose tensors are
    # released first), under a key of its own
    if wl.name == "c2" and not over and not args.no_c3:
        del gc, dg, new_k, new_v, scores, probs
        torch.cuda.empty_cache()
        line["c3"] = million_token_leg(args, K, S, torch)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
