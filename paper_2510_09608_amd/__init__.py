"""MI355X-native streaming KV-cache hot path of StreamingVLM (arXiv 2510.09608).

The product is libsv.so (hand-written HIP for gfx950 behind the C ABI declared in
include/sv.h).  This package is the thin Python binding: it marshals arguments
and nothing else.  PyTorch supplies device memory and streams only.
"""
from .binding import (  # noqa: F401
    SV_DTYPE_BF16, SV_DTYPE_F32, SV_ROPE_1D, SV_ROPE_3D, SV_ROPE_NONE, SV_TEXT, SV_VISION, SV_WINDOW_INF,
    SV_FLAG_GENERIC_KERNELS, SV_FLAG_HOST_LOGIC_ONLY, SV_OPT_CHUNK_SPLITS, SV_OPT_DECODE_TILES_PER_WAVE, SV_OPT_DECODE_SPLITS, SV_OPT_CHUNK_STORE,
    SvConfig, SvChunkIO, SvError, Cache, lib, lib_path,
    sv_attn_chunk, sv_attn_decode, sv_attn_decode_static, sv_cache_append, sv_cache_bytes, sv_cache_create, sv_cache_destroy,
    sv_cache_evict, sv_cache_len, sv_cache_set_option, sv_decode_step, sv_decode_step_layers, sv_stream_step, sv_cache_read_kv, sv_probe_rates, sv_cache_retained, sv_rope_apply, sv_strerror,
)
