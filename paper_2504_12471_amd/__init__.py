"""MI355X-native head-selective ViT block forward/backward (D2FT hot path).

The package is a thin layer over libd2ft.so (hand-written HIP for gfx950):
`binding` mirrors the C ABI of include/d2ft.h one to one, `stack` is the
caller-side loop over blocks.  Importing the package requires the built
library; there is no CPU or PyTorch fallback.
"""
from .binding import (  # noqa: F401
    BF16, F32, FLAG_ACCUM_GRADS, FLAG_DEFER_JOIN, FLAG_GATE_FFN, FLAG_NO_MFMA, FLAG_ONE_STREAM, OP_FULL, OP_FWD, OP_SKIP, SCORE_FISHER, SCORE_MAGNITUDE,
    WEIGHT_FIELDS, BlockDesc, D2ftError, EmbedDesc, HeadDesc,
    d2ft_classifier_fwd_bwd, d2ft_embed_saved_bytes, d2ft_embed_scratch_bytes, d2ft_head_scratch_bytes,
    d2ft_patch_embed_bwd, d2ft_patch_embed_fwd,
    d2ft_block_bwd, d2ft_block_bwd_mb, d2ft_block_fwd, d2ft_block_fwd_mb, d2ft_block_saved_bytes,
    d2ft_block_saved_bytes_mb, d2ft_block_scratch_bytes, d2ft_compact_heads,
    d2ft_knapsack_static_bytes, d2ft_knapsack_workspace_bytes, d2ft_select_knapsack, d2ft_select_knapsack_static,
    d2ft_join, d2ft_sgd_step, d2ft_status_string, d2ft_subnet_scores, d2ft_timing_enable, d2ft_timing_read)
from .stack import BlockStack, make_desc, to_device, torch_dtype  # noqa: F401
