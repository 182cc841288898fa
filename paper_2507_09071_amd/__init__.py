"""MI355X-native sparse prefill attention (BlindSight hot path): thin ctypes binding over
libblindsight.so.  Argument marshalling only — every step of the path runs in the library."""
from .binding import (  # noqa: F401
    BS_BF16, BS_F32, BS_MAP_BIDIR_IMAGES, BS_MAP_PACK_KEYS, BS_MAP_REGROUP_ROWS, DENSE, SINK, INTRA, INTRA_SINK, BlindsightError, TileMap,
    bs_build_tilemap, bs_attn_prefill, bs_attn_prefill_ex, bs_attn_prefill_static, bs_static_scratch_bytes, bs_characterize_prompt, bs_head_sq_error,
    bs_aggregate_head_type, bs_aggregate_layer, bs_alpha_layer, library_path, load_library,
)
