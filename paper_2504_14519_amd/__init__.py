"""MI355X-native sliced causal attention (SlimPipe hot path): thin binding over the C-ABI library."""
from .binding import (  # noqa: F401
    BF16, F32, AttnParams, lib, library_path, slimpipe_attn_fwd, slimpipe_attn_bwd, slimpipe_attn_merge,
    slimpipe_attn_finalize_bf16, slimpipe_attn_workspace_bytes, slimpipe_attn_validate, slimpipe_attn_strerror,
    SlimpipeError, make_params, slimpipe_attn_profile_enable, slimpipe_attn_profile_read, KERNEL_KINDS,
    slimpipe_attn_mfma_rate, slimpipe_attn_fwd_chunked, slimpipe_attn_bwd_chunked, slimpipe_attn_fwd_ranges, slimpipe_attn_init,
    slimpipe_attn_bwd_noalloc, slimpipe_attn_dq_atomic_probe, slimpipe_attn_xcd_rate,
)
