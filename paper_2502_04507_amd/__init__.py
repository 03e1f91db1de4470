"""MI355X-native Sliding Tile Attention forward path (arXiv 2502.04507).

Thin binding over the C-ABI library libsta.so (see include/sta.h): argument
marshalling only -- every step of the path runs in the HIP kernels.  There is
no CPU or PyTorch fallback: if the library is missing, loading fails.
"""
from .binding import (  # noqa: F401
    STA_BF16, STA_F32, StaError, lib_path, load_library, sta_dump_key_tiles, sta_forward, sta_forward_lse,
    sta_kept_flops, sta_key_tile_box, sta_strerror, sta_tile_permute, sta_untile, sta_version,
    sta_window_tokens_to_tiles, sta_workspace_bytes, EXPORTED_SYMBOLS, sta_head_mse_workspace_bytes, sta_head_mse,
    sta_mask_search, sta_attention_recall, sta_block_census, STA_MASK_STA, STA_MASK_NATTEN,
    sta_backward, sta_backward_workspace_bytes, sta_query_tile_box, sta_head_mse_static, sta_forward_general,
)
