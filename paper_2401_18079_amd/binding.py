"""ctypes binding of libkvq.so: argument marshalling only, same names as the C ABI (include/kvq.h)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libkvq.so")
_lib = None


class KvqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = kvq_status_string(status) if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (status {status})")


class _CCache(C.Structure):
    _fields_ = [
        ("bits", C.c_int32), ("head_dim", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32),
        ("k_side_v", C.c_int32), ("loaded", C.c_int32),
        ("cap_tokens", C.c_int64), ("n_tokens_k", C.c_int64), ("n_tokens_v", C.c_int64),
        ("cap_nnz_k", C.c_int64), ("cap_nnz_v", C.c_int64),
        ("rope_base", C.c_float), ("n_sink", C.c_int32),
        ("params", C.c_void_p), ("k_codes", C.c_void_p), ("v_codes", C.c_void_p), ("v_sz", C.c_void_p),
        ("k_ptr", C.c_void_p), ("v_ptr", C.c_void_p),
        ("k_idx", C.c_void_p), ("k_val", C.c_void_p), ("v_idx", C.c_void_p), ("v_val", C.c_void_p),
        ("d_status", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64),
        ("sink_k", C.c_void_p), ("sink_v", C.c_void_p),
        ("nnz_block_shift", C.c_int32), ("reserved0", C.c_int32),
        ("k_idx_blocks", C.c_void_p), ("k_val_blocks", C.c_void_p),
        ("v_idx_blocks", C.c_void_p), ("v_val_blocks", C.c_void_p),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libkvq.so.  There is no fallback: without the built HIP library nothing here works."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it first (python -m paper_2401_18079_amd.build)")
    lib = C.CDLL(_LIB_PATH)
    P, V, I32, I64, F = C.POINTER(_CCache), C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sigs = {
        "kvq_codes_bytes": (I64, [I32, I32, I64]),
        "kvq_params_bytes": (I64, [I32]),
        "kvq_workspace_bytes": (I64, [P, I32]),
        "kvq_status_string": (C.c_char_p, [C.c_int]),
        "kvq_version": (C.c_char_p, []),
        "kvq_stored_signpost": (C.c_float, [C.c_float]),
        "kvq_lut_load": (C.c_int, [P, V, V, V, V, V, V, V]),
        "kvq_quantize_append_k": (C.c_int, [P, V, I32, V]),
        "kvq_quantize_append_v": (C.c_int, [P, V, I32, V]),
        "kvq_quantize_append_kv": (C.c_int, [P, V, V, I32, V]),
        "kvq_qk_matvec": (C.c_int, [P, V, F, V, I64, V]),
        "kvq_pv_matvec": (C.c_int, [P, V, I64, V, V]),
        "kvq_attention_decode": (C.c_int, [P, V, F, V, I64, V, V]),
        "kvq_attention_decode_noalloc": (C.c_int, [P, V, F, V, I64, V, V]),
        "kvq_decode_step": (C.c_int, [P, V, V, V, F, V, I64, V, V]),
        "kvq_decode_step_launches": (I32, [P]),
        "kvq_softmax_workspace_bytes": (I64, [I32, I64]),
        "kvq_softmax_f32": (C.c_int, [V, I64, V, I64, I32, I64, V, I64, V]),
        "kvq_calibrate_key_channels": (C.c_int, [V, I32, I32, F, V, V, V, V, V]),
        "kvq_calibrate_workspace_bytes": (I64, []),
        "kvq_calibrate_nuq": (C.c_int, [V, V, I64, I32, I32, V, V, I64, V]),
        "kvq_fp16_qk_matvec": (C.c_int, [V, I64, I32, I32, V, F, V, I64, V]),
        "kvq_fp16_pv_workspace_bytes": (I64, [I32, I64]),
        "kvq_fp16_pv_matvec": (C.c_int, [V, I64, I32, I32, V, I64, V, V, I64, V]),
        "kvq_stream_read_workspace_bytes": (I64, []),
        "kvq_stream_read": (C.c_int, [V, I64, V, I64, V]),
        "kvq_event_create": (C.c_int, [C.POINTER(V)]),
        "kvq_event_record": (C.c_int, [V, V]),
        "kvq_event_elapsed_ms": (C.c_int, [V, V, C.POINTER(F)]),
        "kvq_event_destroy": (C.c_int, [V]),
        "kvq_profile_enable": (C.c_int, [I32]),
        "kvq_profile_last_ms": (C.c_int, [I32, C.POINTER(F)]),
        "kvq_profile_count": (C.c_int, [I32, C.POINTER(I64)]),
        "kvq_profile_read_ms": (C.c_int, [I32, I64, C.POINTER(F)]),
        "kvq_profile_span_buffer_bytes": (I64, []),
        "kvq_profile_set_span_buffer": (C.c_int, [V, I64]),
        "kvq_profile_span_us": (C.c_int, [I32, I64, C.POINTER(F)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTED_SYMBOLS = [
    "kvq_codes_bytes", "kvq_params_bytes", "kvq_workspace_bytes", "kvq_status_string", "kvq_version",
    "kvq_lut_load", "kvq_stored_signpost", "kvq_quantize_append_k", "kvq_quantize_append_v", "kvq_quantize_append_kv",
    "kvq_qk_matvec", "kvq_pv_matvec",
    "kvq_attention_decode", "kvq_attention_decode_noalloc", "kvq_decode_step", "kvq_decode_step_launches", "kvq_softmax_workspace_bytes", "kvq_softmax_f32", "kvq_fp16_qk_matvec", "kvq_fp16_pv_workspace_bytes",
    "kvq_fp16_pv_matvec", "kvq_event_create", "kvq_event_record", "kvq_event_elapsed_ms", "kvq_event_destroy",
    "kvq_profile_enable", "kvq_profile_last_ms", "kvq_profile_count", "kvq_profile_read_ms",
    "kvq_profile_span_buffer_bytes", "kvq_profile_set_span_buffer", "kvq_profile_span_us", "kvq_calibrate_workspace_bytes", "kvq_calibrate_nuq",
    "kvq_calibrate_key_channels", "kvq_stream_read_workspace_bytes", "kvq_stream_read",
]


_span_buffer = None


def kvq_profile_enable(on: bool, spans: bool = False, events: bool = True):
    """Switch the per-kernel timing aid on or off.  spans: also (or, with events=False, only) take each
    dense kernel's own first-start-to-last-end span; the device buffer they land in is allocated here."""
    global _span_buffer
    lib = load_library()
    if not on:
        _check(lib.kvq_profile_enable(0), "kvq_profile_enable")
        return
    _check(lib.kvq_profile_enable(0), "kvq_profile_enable")
    if spans and _span_buffer is None:
        _span_buffer = torch.zeros(int(lib.kvq_profile_span_buffer_bytes()) // 8, dtype=torch.int64, device="cuda")
    _check(lib.kvq_profile_set_span_buffer(_span_buffer.data_ptr() if spans else None,
                                           _span_buffer.numel() * 8 if spans else 0), "kvq_profile_set_span_buffer")
    _check(lib.kvq_profile_enable(1 if events else 3), "kvq_profile_enable")


def kvq_profile_read_all_spans_us(which: int):
    """Spans (us) of every dense-kernel launch recorded since kvq_profile_enable(True, spans=True)."""
    lib = load_library()
    n = C.c_int64()
    _check(lib.kvq_profile_count(which, C.byref(n)), "kvq_profile_count")
    out, us = [], C.c_float()
    for call in range(max(0, n.value - 256), n.value):
        _check(lib.kvq_profile_span_us(which, call, C.byref(us)), "kvq_profile_span_us")
        out.append(float(us.value))
    return out


def kvq_profile_read_all_us(which: int):
    """Durations (us) of every dense-kernel launch recorded since kvq_profile_enable(True) (at most the last 256)."""
    lib = load_library()
    n = C.c_int64()
    _check(lib.kvq_profile_count(which, C.byref(n)), "kvq_profile_count")
    out, ms = [], C.c_float()
    for call in range(max(0, n.value - 256), n.value):
        _check(lib.kvq_profile_read_ms(which, call, C.byref(ms)), "kvq_profile_read_ms")
        out.append(float(ms.value) * 1e3)
    return out


def kvq_profile_last_ms(which: int) -> float:
    ms = C.c_float()
    _check(load_library().kvq_profile_last_ms(which, C.byref(ms)), "kvq_profile_last_ms")
    return float(ms.value)


def _stream_ptr(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise KvqError(status, where)


def kvq_status_string(status: int) -> str:
    return load_library().kvq_status_string(int(status)).decode()


def kvq_version() -> str:
    return load_library().kvq_version().decode()


def kvq_stored_signpost(x: float) -> float:
    return float(load_library().kvq_stored_signpost(float(x)))


def kvq_codes_bytes(bits: int, n_kv_heads: int, cap_tokens: int) -> int:
    return int(load_library().kvq_codes_bytes(bits, n_kv_heads, cap_tokens))


def kvq_params_bytes(n_kv_heads: int) -> int:
    return int(load_library().kvq_params_bytes(n_kv_heads))


def kvq_workspace_bytes(cache: "KvqCache", max_append: int) -> int:
    return int(load_library().kvq_workspace_bytes(C.byref(cache.c), max_append))


class KvqCache:
    """Device buffers of one layer's cache for one sequence (torch tensors) plus the C descriptor."""

    def __init__(self, bits, n_kv_heads, n_q_heads, cap_tokens, k_side_v, rope_base, cap_nnz_k, cap_nnz_v=None,
                 max_append=4096, device="cuda:0", n_sink=0, nnz_block_entries=None, nnz_table_slots=4096):
        """nnz_block_entries: None for flat outlier arrays of cap_nnz_k / cap_nnz_v entries; a power of two
        (1024 .. 2^30) for blocked storage, where the capacities are rounded up to whole blocks and
        ensure_nnz_room() adds blocks without copying.  nnz_table_slots: blocks each table can list."""
        load_library()
        dev = torch.device(device)
        D = n_kv_heads * 128
        if cap_nnz_v is None:
            cap_nnz_v = max(8, cap_tokens * 2 * k_side_v)
        cap_nnz_k = max(8, int(cap_nnz_k))
        z = lambda n, dt: torch.zeros(int(n), dtype=dt, device=dev)
        self.params = z(kvq_params_bytes(n_kv_heads), torch.uint8)
        nbytes = kvq_codes_bytes(bits, n_kv_heads, cap_tokens)
        self.k_codes, self.v_codes = z(nbytes, torch.uint8), z(nbytes, torch.uint8)
        self.v_sz = z(cap_tokens * 2, torch.int16)
        self.k_ptr, self.v_ptr = z(cap_tokens + 1, torch.int32), z(cap_tokens + 1, torch.int32)
        self.block_entries = int(nnz_block_entries or 0)
        if self.block_entries:
            be = self.block_entries
            assert be & (be - 1) == 0 and 1 << 10 <= be <= 1 << 30, "block size: a power of two in [2^10, 2^30]"
            cap_nnz_k, cap_nnz_v = -(-cap_nnz_k // be) * be, -(-int(cap_nnz_v) // be) * be
            assert max(cap_nnz_k, cap_nnz_v) // be <= nnz_table_slots
            self.k_idx = self.k_val = self.v_idx = self.v_val = None
            self.blocks = {n: [z(be, torch.int16) for _ in range(cap // be)]
                           for n, cap in (("k_idx", cap_nnz_k), ("k_val", cap_nnz_k), ("v_idx", cap_nnz_v), ("v_val", cap_nnz_v))}
            self.tables = {n: z(nnz_table_slots, torch.int64) for n in self.blocks}
            for n, bl in self.blocks.items():
                self.tables[n][:len(bl)] = torch.tensor([b.data_ptr() for b in bl], dtype=torch.int64)
        else:
            self.k_idx, self.k_val = z(cap_nnz_k, torch.int16), z(cap_nnz_k, torch.int16)
            self.v_idx, self.v_val = z(cap_nnz_v, torch.int16), z(cap_nnz_v, torch.int16)
        self.d_status = z(4, torch.int32)
        # attention-sink tokens: the first n_sink tokens are also kept in fp16
        self.sink_k, self.sink_v = z(max(1, n_sink) * D, torch.int16), z(max(1, n_sink) * D, torch.int16)
        c = _CCache()
        c.bits, c.head_dim, c.n_kv_heads, c.n_q_heads = bits, 128, n_kv_heads, n_q_heads
        c.k_side_v, c.loaded = k_side_v, 0
        c.cap_tokens, c.n_tokens_k, c.n_tokens_v = cap_tokens, 0, 0
        c.cap_nnz_k, c.cap_nnz_v = cap_nnz_k, int(cap_nnz_v)
        c.rope_base = float(rope_base)
        c.n_sink = int(n_sink)
        for name in ("params", "k_codes", "v_codes", "v_sz", "k_ptr", "v_ptr", "d_status", "sink_k", "sink_v"):
            setattr(c, name, getattr(self, name).data_ptr())
        for name in ("k_idx", "k_val", "v_idx", "v_val"):
            if self.block_entries:
                setattr(c, name + "_blocks", self.tables[name].data_ptr())
            else:
                setattr(c, name, getattr(self, name).data_ptr())
        c.nnz_block_shift = self.block_entries.bit_length() - 1 if self.block_entries else 0
        self.c = c
        self.D, self.device = D, dev
        self.workspace = z(int(load_library().kvq_workspace_bytes(C.byref(c), max_append)), torch.uint8)
        c.workspace, c.workspace_bytes = self.workspace.data_ptr(), self.workspace.numel()

    @property
    def n_tokens_k(self):
        return int(self.c.n_tokens_k)

    @property
    def n_tokens_v(self):
        return int(self.c.n_tokens_v)

    def status(self) -> int:
        return int(self.d_status[0].item())

    # Growing the sparse arrays.  The library never allocates: capacity is a field of the descriptor and
    # the owner of the memory grows it between calls.  With blocked storage (paper App. "Limitations":
    # the outlier storage allocated in blocks, so that appending a token copies nothing already
    # stored) growing is one new block per array and one 8-byte store into each block table; with flat
    # arrays it is a new, larger allocation and a copy of the entries in use, by NNZ_BLOCK entries at a
    # time so that the copies are amortised.
    NNZ_BLOCK = 1 << 20

    def nnz_used(self):
        """(Key, Value) outlier entries stored so far.  Reads two device words: synchronises."""
        k = int(self.k_ptr[self.n_tokens_k].item()) & 0xFFFFFFFF
        v = int(self.v_ptr[self.n_tokens_v].item()) & 0xFFFFFFFF
        return k, v

    def sparse_entries(self, side: str, n: int):
        """The first n (index, value) entries of side "k" or "v" as two int16 tensors, whatever the layout."""
        if not self.block_entries:
            return getattr(self, side + "_idx")[:n], getattr(self, side + "_val")[:n]
        return (torch.cat(self.blocks[side + "_idx"])[:n], torch.cat(self.blocks[side + "_val"])[:n])

    def ensure_nnz_room(self, extra_k: int, extra_v: int, block: int = None) -> bool:
        """Make room for `extra_k` / `extra_v` more outlier entries (worst case of the next appends: every
        element of a Key token can be an outlier, a Value token has exactly 2 * k_side_v).  Blocked
        storage: adds blocks, copies nothing.  Flat arrays: reallocates in steps of `block` entries and
        copies the entries in use.  Returns True if anything grew."""
        used_k, used_v = self.nnz_used()
        grew = False
        if self.block_entries:
            be = self.block_entries
            for used, extra, cap_name, names in ((used_k, extra_k, "cap_nnz_k", ("k_idx", "k_val")),
                                                 (used_v, extra_v, "cap_nnz_v", ("v_idx", "v_val"))):
                while used + int(extra) > getattr(self.c, cap_name):
                    n = getattr(self.c, cap_name) // be
                    if n >= self.tables[names[0]].numel() or (n + 1) * be >= 1 << 31:
                        raise KvqError(3, "ensure_nnz_room")
                    for name in names:
                        blk = torch.zeros(be, dtype=torch.int16, device=self.device)
                        self.blocks[name].append(blk)
                        self.tables[name][n] = blk.data_ptr()      # one 8-byte store, ordered on the stream
                    setattr(self.c, cap_name, (n + 1) * be)
                    grew = True
            return grew
        block = int(block or self.NNZ_BLOCK)
        for used, extra, cap_name, names in ((used_k, extra_k, "cap_nnz_k", ("k_idx", "k_val")),
                                             (used_v, extra_v, "cap_nnz_v", ("v_idx", "v_val"))):
            need = used + int(extra)
            if need <= getattr(self.c, cap_name):
                continue
            if need >= 1 << 31:
                raise KvqError(3, "ensure_nnz_room")            # the mat-vec kernels address entries with 32-bit byte offsets
            cap = min((need + block - 1) // block * block, (1 << 31) - 1)
            for name in names:
                old = getattr(self, name)
                new_t = torch.zeros(cap, dtype=old.dtype, device=old.device)
                new_t[:used] = old[:used]
                setattr(self, name, new_t)
                setattr(self.c, name, new_t.data_ptr())
            setattr(self.c, cap_name, cap)
            grew = True
        if grew:
            torch.cuda.synchronize(self.device)                 # the old arrays are released after the copies
        return grew


def _host_u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def kvq_lut_load(cache: KvqCache, lut_k, lut_v, s_k, z_k, lo_k, hi_k, stream=None):
    lk = np.ascontiguousarray(lut_k, dtype=np.float32)
    lv = np.ascontiguousarray(lut_v, dtype=np.float32)
    arrs = [_host_u16(a) for a in (s_k, z_k, lo_k, hi_k)]
    assert lk.size == 1 << cache.c.bits and lv.size == lk.size and all(a.size == cache.D for a in arrs)
    st = load_library().kvq_lut_load(C.byref(cache.c), lk.ctypes.data, lv.ctypes.data,
                                     *[a.ctypes.data for a in arrs], _stream_ptr(stream))
    _check(st, "kvq_lut_load")


def _fp16_rows(cache: KvqCache, x: torch.Tensor):
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.shape[1] == cache.D and x.is_contiguous()
    return x


def kvq_quantize_append_k(cache: KvqCache, k_new: torch.Tensor, stream=None):
    x = _fp16_rows(cache, k_new)
    _check(load_library().kvq_quantize_append_k(C.byref(cache.c), x.data_ptr(), x.shape[0], _stream_ptr(stream)),
           "kvq_quantize_append_k")


def kvq_quantize_append_v(cache: KvqCache, v_new: torch.Tensor, stream=None):
    x = _fp16_rows(cache, v_new)
    _check(load_library().kvq_quantize_append_v(C.byref(cache.c), x.data_ptr(), x.shape[0], _stream_ptr(stream)),
           "kvq_quantize_append_v")


def kvq_quantize_append_kv(cache: KvqCache, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
    xk, xv = _fp16_rows(cache, k_new), _fp16_rows(cache, v_new)
    assert xk.shape[0] == xv.shape[0]
    _check(load_library().kvq_quantize_append_kv(C.byref(cache.c), xk.data_ptr(), xv.data_ptr(), xk.shape[0],
                                                 _stream_ptr(stream)), "kvq_quantize_append_kv")


def kvq_qk_matvec(cache: KvqCache, q_rot: torch.Tensor, scale: float, scores: torch.Tensor, stream=None):
    assert q_rot.is_cuda and q_rot.dtype == torch.float32 and q_rot.is_contiguous()
    assert q_rot.shape == (cache.c.n_q_heads, 128)
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.dim() == 2 and scores.stride(1) == 1
    assert scores.shape[0] == cache.c.n_q_heads
    _check(load_library().kvq_qk_matvec(C.byref(cache.c), q_rot.data_ptr(), float(scale), scores.data_ptr(),
                                        scores.stride(0), _stream_ptr(stream)), "kvq_qk_matvec")


def kvq_pv_matvec(cache: KvqCache, probs: torch.Tensor, out: torch.Tensor, stream=None):
    assert probs.is_cuda and probs.dtype == torch.float32 and probs.dim() == 2 and probs.stride(1) == 1
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == (cache.c.n_q_heads, 128)
    _check(load_library().kvq_pv_matvec(C.byref(cache.c), probs.data_ptr(), probs.stride(0), out.data_ptr(),
                                        _stream_ptr(stream)), "kvq_pv_matvec")


def kvq_attention_decode(cache: KvqCache, q_rot: torch.Tensor, scale: float, scores: torch.Tensor, out: torch.Tensor,
                         stream=None):
    assert q_rot.is_cuda and q_rot.dtype == torch.float32 and q_rot.is_contiguous()
    assert q_rot.shape == (cache.c.n_q_heads, 128)
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.dim() == 2 and scores.stride(1) == 1
    assert scores.shape[0] == cache.c.n_q_heads
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == (cache.c.n_q_heads, 128)
    _check(load_library().kvq_attention_decode(C.byref(cache.c), q_rot.data_ptr(), float(scale), scores.data_ptr(),
                                               scores.stride(0), out.data_ptr(), _stream_ptr(stream)),
           "kvq_attention_decode")


def kvq_decode_step(cache: KvqCache, k_new: torch.Tensor, v_new: torch.Tensor, q_rot: torch.Tensor, scale: float,
                    scores: torch.Tensor, out: torch.Tensor, stream=None):
    """Append one token's Key and Value, then the fused attention over the cache that ends with it."""
    k, v = _fp16_rows(cache, k_new), _fp16_rows(cache, v_new)
    assert k.shape[0] == 1 and v.shape[0] == 1
    assert q_rot.is_cuda and q_rot.dtype == torch.float32 and q_rot.is_contiguous()
    assert q_rot.shape == (cache.c.n_q_heads, 128)
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.dim() == 2 and scores.stride(1) == 1
    assert scores.shape[0] == cache.c.n_q_heads
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == (cache.c.n_q_heads, 128)
    _check(load_library().kvq_decode_step(C.byref(cache.c), k.data_ptr(), v.data_ptr(), q_rot.data_ptr(), float(scale),
                                          scores.data_ptr(), scores.stride(0), out.data_ptr(), _stream_ptr(stream)),
           "kvq_decode_step")


def kvq_decode_step_launches(cache: KvqCache) -> int:
    return int(load_library().kvq_decode_step_launches(C.byref(cache.c)))


def kvq_attention_decode_noalloc(cache: KvqCache, q_rot: torch.Tensor, scale: float, scores: torch.Tensor,
                                 out: torch.Tensor, stream=None):
    """kvq_attention_decode on the library's static scratch: cache.workspace is not used."""
    assert q_rot.is_cuda and q_rot.dtype == torch.float32 and q_rot.is_contiguous()
    assert q_rot.shape == (cache.c.n_q_heads, 128)
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.dim() == 2 and scores.stride(1) == 1
    assert scores.shape[0] == cache.c.n_q_heads
    assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and out.shape == (cache.c.n_q_heads, 128)
    _check(load_library().kvq_attention_decode_noalloc(C.byref(cache.c), q_rot.data_ptr(), float(scale),
                                                       scores.data_ptr(), scores.stride(0), out.data_ptr(),
                                                       _stream_ptr(stream)), "kvq_attention_decode_noalloc")


def kvq_softmax_f32(x: torch.Tensor, probs: torch.Tensor, n_cols: int, workspace: torch.Tensor, stream=None):
    assert x.is_cuda and x.dtype == torch.float32 and x.stride(1) == 1 and probs.stride(1) == 1
    _check(load_library().kvq_softmax_f32(x.data_ptr(), x.stride(0), probs.data_ptr(), probs.stride(0), x.shape[0],
                                          int(n_cols), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream_ptr(stream)), "kvq_softmax_f32")


def kvq_calibrate_key_channels(k_cal: torch.Tensor, outlier_fraction: float, stream=None):
    """Per-channel Key constants (s, z, lo, hi) as fp16 numpy arrays, from calibration Keys [T][D] on the GPU."""
    assert k_cal.is_cuda and k_cal.dtype == torch.float16 and k_cal.dim() == 2 and k_cal.is_contiguous()
    T, D = k_cal.shape
    outs = [torch.empty(D, dtype=torch.int16, device=k_cal.device) for _ in range(4)]
    _check(load_library().kvq_calibrate_key_channels(k_cal.data_ptr(), T, D, float(outlier_fraction),
                                                     *[o.data_ptr() for o in outs], _stream_ptr(stream)),
           "kvq_calibrate_key_channels")
    return tuple(o.cpu().numpy().view(np.float16) for o in outs)


def kvq_calibrate_nuq(x_norm: torch.Tensor, w: torch.Tensor, bits: int, iters: int, init, stream=None) -> np.ndarray:
    """Signposts of the non-uniform datatype from normalised calibration values and their weights."""
    assert x_norm.is_cuda and w.is_cuda and x_norm.dtype == torch.float32 and w.dtype == torch.float32
    assert x_norm.dim() == 1 and x_norm.is_contiguous() and w.is_contiguous() and w.shape == x_norm.shape
    lib = load_library()
    c = np.ascontiguousarray(np.asarray(init, dtype=np.float32).copy())
    assert c.shape == (1 << bits,)
    ws = torch.empty(int(lib.kvq_calibrate_workspace_bytes()), dtype=torch.uint8, device=x_norm.device)
    _check(lib.kvq_calibrate_nuq(x_norm.data_ptr(), w.data_ptr(), x_norm.numel(), int(bits), int(iters),
                                 c.ctypes.data_as(C.c_void_p), ws.data_ptr(), ws.numel(), _stream_ptr(stream)),
           "kvq_calibrate_nuq")
    return c


def kvq_softmax_workspace_bytes(n_rows: int, n_cols: int) -> int:
    return int(load_library().kvq_softmax_workspace_bytes(n_rows, n_cols))


def kvq_fp16_qk_matvec(k16: torch.Tensor, n_kv_heads: int, n_q_heads: int, q: torch.Tensor, scale: float,
                       scores: torch.Tensor, stream=None):
    assert k16.dtype == torch.float16 and k16.is_contiguous() and k16.shape[1] == n_kv_heads * 128
    _check(load_library().kvq_fp16_qk_matvec(k16.data_ptr(), k16.shape[0], n_kv_heads, n_q_heads, q.data_ptr(),
                                             float(scale), scores.data_ptr(), scores.stride(0), _stream_ptr(stream)),
           "kvq_fp16_qk_matvec")


def kvq_fp16_pv_workspace_bytes(n_q_heads: int, L: int) -> int:
    return int(load_library().kvq_fp16_pv_workspace_bytes(n_q_heads, L))


def kvq_fp16_pv_matvec(v16: torch.Tensor, n_kv_heads: int, n_q_heads: int, probs: torch.Tensor, out: torch.Tensor,
                       workspace: torch.Tensor, stream=None):
    assert v16.dtype == torch.float16 and v16.is_contiguous() and v16.shape[1] == n_kv_heads * 128
    _check(load_library().kvq_fp16_pv_matvec(v16.data_ptr(), v16.shape[0], n_kv_heads, n_q_heads, probs.data_ptr(),
                                             probs.stride(0), out.data_ptr(), workspace.data_ptr(),
                                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "kvq_fp16_pv_matvec")


def kvq_stream_read(buf: torch.Tensor, workspace: torch.Tensor, stream=None):
    """Reads `buf` once (the streaming-read reference); per-workgroup checksums land in `workspace` (uint32)."""
    assert buf.is_cuda and buf.is_contiguous() and workspace.is_cuda and workspace.is_contiguous()
    _check(load_library().kvq_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), workspace.data_ptr(),
                                          workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "kvq_stream_read")


def kvq_stream_read_workspace_bytes() -> int:
    return int(load_library().kvq_stream_read_workspace_bytes())


class HipEventTimer:
    """HIP events recorded on the stream the kernels are launched on (kvq_event_* of the C ABI)."""

    def __init__(self):
        lib = load_library()
        self._a, self._b = C.c_void_p(), C.c_void_p()
        _check(lib.kvq_event_create(C.byref(self._a)), "kvq_event_create")
        _check(lib.kvq_event_create(C.byref(self._b)), "kvq_event_create")

    def start(self, stream=None):
        _check(load_library().kvq_event_record(self._a, _stream_ptr(stream)), "kvq_event_record")

    def stop(self, stream=None):
        _check(load_library().kvq_event_record(self._b, _stream_ptr(stream)), "kvq_event_record")

    def elapsed_ms(self) -> float:
        ms = C.c_float()
        _check(load_library().kvq_event_elapsed_ms(self._a, self._b, C.byref(ms)), "kvq_event_elapsed_ms")
        return float(ms.value)

    def __del__(self):
        try:
            lib = load_library()
            lib.kvq_event_destroy(self._a)
            lib.kvq_event_destroy(self._b)
        except Exception:
            pass
