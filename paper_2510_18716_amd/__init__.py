"""MI355X-native SSD compressed decode attention: thin Python binding over libssd_hip.so.

The binding only marshals arguments (tensor pointers, sizes, the current HIP stream); every step
of the path runs in the library's HIP kernels.  There is no CPU or PyTorch fallback: importing
this package without the built library raises.
"""
from .binding import (  # noqa: F401
    SSD_BF16, SSD_F32, SSD_SEMANTIC, SSD_SPATIAL,
    SSD_ERR_HIP, SSD_ERR_INVALID_ARG, SSD_ERR_LAYER_RANGE, SSD_ERR_ORDER, SSD_ERR_STAGE_OVERFLOW, SSD_OK,
    Cache, SsdConfig, SsdError, lib, lib_path,
    ssd_append_token, ssd_cache_bytes, ssd_cfg_mix, ssd_classify_heads, ssd_compress_kv, ssd_decode_attn, ssd_decode_step,
    SSD_ROPE_HALF, SSD_ROPE_INTERLEAVED, ssd_decode_step_rope,
    SSD_MAX_SPLIT, SSD_SPLIT_FORK, SSD_SPLIT_JOIN, ssd_decode_step_split, ssd_decode_step_split_rope, stream_array,
    ssd_dense_decode_attn, ssd_dense_decode_attn_static, SSD_DENSE_STATIC_SCRATCH_BYTES, ssd_dense_workspace_bytes, ssd_last_error, ssd_prefill_scores, ssd_version,
)
