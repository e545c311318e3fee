"""kvq: KVQuant decode-time hot path on AMD MI355X (gfx950).

Thin Python binding over the C-ABI library in csrc/ (see include/kvq.h).  PyTorch is used only for
device memory and streams; every step of the path runs in the HIP kernels.
"""
from .binding import (  # noqa: F401
    KvqError, KvqCache, lib_path, load_library,
    kvq_lut_load, kvq_quantize_append_k, kvq_quantize_append_v, kvq_quantize_append_kv, kvq_qk_matvec, kvq_pv_matvec, kvq_attention_decode, kvq_attention_decode_noalloc, kvq_decode_step, kvq_decode_step_launches,
    kvq_softmax_f32, kvq_fp16_qk_matvec, kvq_fp16_pv_matvec, kvq_codes_bytes, kvq_params_bytes,
    kvq_workspace_bytes, kvq_status_string, kvq_version, kvq_stored_signpost, HipEventTimer, kvq_profile_enable, kvq_profile_last_ms, kvq_profile_read_all_us, kvq_profile_read_all_spans_us,
    kvq_calibrate_nuq, kvq_calibrate_key_channels, kvq_stream_read,
)
