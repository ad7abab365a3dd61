"""MI355X-native paged FP8 grouped-query decode attention (the LLM-CoOpt hot path).

The product is ``libcoopt_attn.so`` (hand-written HIP for gfx950 behind the C ABI declared in
``include/coopt_attn.h``).  This package is the thin Python binding over it: argument marshalling
only.  There is no CPU fallback: importing works anywhere, calling needs the built library and a GPU.
"""
from .binding import (  # noqa: F401
    COOPT_KV_E4M3, COOPT_KV_E5M2, COOPT_KV_FP16, COOPT_SCALE_BLOCK, COOPT_SCALE_STATIC,
    COOPT_SCALE_TOKEN, CooptError, DecodePlan, Shape, decode_schedule_bytes,
    decode_builtin_workspace_bytes, decode_schedule_prepare, decode_workspace_bytes, default_decode_plan, gather_cached_kv,
    kv_cache_write_fp16, kv_cache_write_fp8, kv_cache_write_fp8_scaled, kv_cache_write_skipset, lib_path, load_library,
    make_decode_plan, paged_gqa_decode, paged_gqa_decode_merge, paged_gqa_decode_noalloc, paged_gqa_decode_partitioned,
    paged_gqa_decode_scheduled, paged_gqa_decode_split, paged_gqa_decode_step,
    paged_gqa_prefill_chunk, paged_gqa_prefill_chunk_ws, paged_gqa_reduce, prefill_workspace_bytes,
    status_string)
