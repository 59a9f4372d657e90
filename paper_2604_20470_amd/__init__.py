"""MI355X-native DynamicRad attention hot path: thin Python binding over the C-ABI library.

The three stages (block scores -> mask -> block-sparse attention) run entirely in
the hand-written gfx950 kernels of ``libdynamicrad.so``; this package only marshals
torch device pointers and streams into the C calls declared in include/dynamicrad.h.
There is no CPU fallback: if the library is not built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    Context, DRError, MaskParams, Shape, dr_block_scores, dr_build_mask, dr_class_map, dr_mask_capacity,
    dr_build_mask_tokens, dr_proxy_loss, dr_static_ratio_for_sparsity, dr_clock_probe, dr_mfma_probe, dr_mfma_mix_probe, dr_sparse_attn_fwd, dr_sparse_attn_fwd_static, dr_token_scores, lib_path, load_library, shape_of, version,
    MODE_STATIC, MODE_DYNAMIC, MODE_ZSCORE, MODE_UNIFORM, CLASS_NONE, CLASS_NEAR, CLASS_FAR, CLASS_FORCED,
)
