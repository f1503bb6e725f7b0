"""MI355X-native EarlyTom vision-encoder hot path: Python binding over libearlytom.so.

Every computation happens in the HIP library; this package only marshals arguments
(torch is used for device memory and streams).  There is no CPU fallback: importing
the binding's functions without a built library raises.
"""
from .binding import (  # noqa: F401
    EtError, load_library, library_path,
    et_keep_count, et_last_error, et_merge_workspace_bytes, et_merge_select,
    et_merge_select_policy, et_encode_clip_policy, et_encode_clip_multi, et_attention_scores,
    et_frame_similarity, et_segment_scan, et_segment_mean, et_topk_select, et_compact_tokens,
    et_layernorm, et_gemm_bf16, et_attention, et_attention_uniform, et_merge_select_static,
    et_encoder_block_qkv,
    et_encoder_create, et_encoder_destroy, et_workspace_bytes, et_encode_clip,
    et_profile_enable, et_profile_read, et_kernel_name, et_merge_profile_enable, et_merge_profile_read,
    Encoder, Projector, KERNEL_KINDS,
)
