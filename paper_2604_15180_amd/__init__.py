"""MI355X-native fused alpha-entmax attention (AdaSplash-2 hot path): thin binding over the
C ABI in include/entmax_attn.h.  All arithmetic runs in the HIP library; this package only
marshals arguments.  There is no CPU fallback: without the built library, calls raise."""
from .binding import (  # noqa: F401
    EntmaxAttnError, entmax_attn_bwd, entmax_attn_fwd, entmax_attn_histogram_bins,
    entmax_attn_mask_tile, entmax_attn_strerror, entmax_attn_workspace_bytes, lib, lib_path,
    read_stats, STAT_NAMES, entmax_attn_timer_enable, entmax_attn_timer_read, entmax_attn_mfma_probe,
    entmax_attn_decode, entmax_attn_decode_workspace_bytes, entmax_attn_gather_enable,
    entmax_attn_decode_static, entmax_attn_decode_static_max_bytes, entmax_attn_fwd_histogram_bounds,
    entmax_attn_right_edge_enable, entmax_attn_coissue_probe,
)
