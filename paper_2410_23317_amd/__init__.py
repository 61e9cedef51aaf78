"""MI355X-native VL-Cache hot path: hand-written HIP kernels behind a C-ABI (include/vlcache.h)
and a thin ctypes binding with the same names."""
from .binding import (  # noqa: F401
    VLC_BF16, VLC_ERR_CAPACITY, VLC_ERR_DTYPE, VLC_ERR_HIP, VLC_ERR_INVALID_ARG, VLC_ERR_SHAPE,
    VLC_ERR_UNIMPLEMENTED, VLC_F32, VLC_OK, Cache, VlcError, lib, make_shape, vlc_allocate, vlc_cache_bytes,
    vlc_cache_bytes_fp8, vlc_cache_bytes_opt, vlc_cache_create, vlc_cache_create_opt, vlc_cache_options, make_options, VLC_SHAPE_SCORE_PLAIN_ALU, vlc_cache_create_fp8, vlc_cache_hit_rate, vlc_cache_layout, vlc_cache_status, vlc_decode_attn, vlc_decode_attn_steps, vlc_last_error_string, vlc_probe_read_stream, vlc_score,
    vlc_score_from_stats, vlc_score_static, vlc_score_static_max_workspace, vlc_window_attn, vlc_window_attn_workspace_bytes,
    vlc_shape, vlc_sparsity, vlc_topk_compact, vlc_topk_compact_recent_frac, vlc_version, vlc_workspace_bytes,
)
