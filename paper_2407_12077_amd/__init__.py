"""MI355X-native WKV6 prefill: HIP kernels behind a C ABI, with a thin ctypes binding."""
from .binding import (  # noqa: F401
    WKV6_DTYPE_BF16, WKV6_DTYPE_F32, Wkv6Error, load, status_string, wkv6_append_bf16, wkv6_decode_bf16,
    wkv6_decay_lora_input_bf16, wkv6_finch_c2_append_bf16, wkv6_finch_c2_decode_bf16, wkv6_finch_c2_prefill_bf16,
    wkv6_finch_c2_prefill_bf16_moments, wkv6_finch_c2_prefill_bf16_split, wkv6_finch_c2_prefill_lora_bf16, wkv6_layernorm_apply_bf16, wkv6_layernorm_finalize,
    wkv6_key_compress_bf16,
    wkv6_finch_c2_prefill_bf16_f32out, wkv6_finch_c2_prefill_bf16_strided, wkv6_prefill_bf16,
    wkv6_prefill_bf16_f32out, wkv6_prefill_bf16_recurrent, wkv6_prefill_lora_bf16, wkv6_prefill_bf16_split, wkv6_prefill_bf16_split_noalloc,
    wkv6_prefill_bf16_strided, wkv6_prefill_f32, wkv6_split_segments, wkv6_split_workspace_bytes,
    wkv6_arena_layout, wkv6_version)
