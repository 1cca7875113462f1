"""MI355X-native decode attention over a CommVQ-compressed KV cache.

Thin ctypes binding over ``libcommvq.so`` (hand-written HIP for gfx950).  The
functions carry the names of the C entry points in ``include/commvq.h`` and only
marshal arguments; every step of the path runs in the library's kernels.  There
is no CPU fallback: without the built library, or without a GPU, calls raise.
"""
from .binding import (  # noqa: F401
    COMMVQ_BF16,
    COMMVQ_F32,
    COMMVQ_KEYS_INDEXED,
    COMMVQ_KEYS_PAIRED,
    CommVQError,
    Config,
    Handle,
    Plan,
    Positions,
    commvq_create,
    commvq_create_planner,
    commvq_decode_attn,
    commvq_decode_attn_static,
    commvq_destroy,
    commvq_em_shared_workspace_bytes,
    commvq_em_step,
    commvq_em_step_shared,
    commvq_em_workspace_bytes,
    commvq_encode_keys,
    commvq_encode_values,
    commvq_encoder_prepare,
    commvq_encoder_table_bytes,
    commvq_forget_packed_key_codebooks,
    commvq_pack_key_codebooks,
    commvq_packed_key_codebook_bytes,
    commvq_plan_query,
    commvq_profile_enable,
    commvq_profile_read,
    commvq_stage_bins,
    commvq_stage_output,
    commvq_stage_scores,
    commvq_static_scratch_bytes,
    commvq_status_string,
    commvq_validate_config,
    commvq_value_encoder_prepare,
    commvq_value_encoder_table_bytes,
    commvq_workspace_bytes,
    library_path,
    load_library,
)
