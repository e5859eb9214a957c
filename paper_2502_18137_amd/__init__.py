"""MI355X-native SpargeAttn hot path: thin Python binding over the C-ABI library libsparge.so.

Importing the package does not load the library; the first call does, and fails loudly if the
library has not been built (python -m paper_2502_18137_amd.build).
"""
from .binding import (  # noqa: F401
    AttnKernelTimer,
    SpargeError,
    library_path,
    load_library,
    sparge_attn,
    sparge_attn_quantized,
    sparge_attn_tiled,
    sparge_mask_to_lut,
    sparge_v_tiles,
    sparge_forward,
    sparge_predict,
    sparge_predict_static,
    STATIC_SCRATCH_BYTES,
    sparge_hilbert_order,
    sparge_item_order,
    sparge_permute_tokens,
    sparge_quantize,
    sparge_rel_l1,
    sparge_tune,
    sparge_version,
    sparge_workspace_bytes,
    tensor_from_numpy,
    REF_SLACK_LOG2,
    REF_SLACK_LOG2_FP8,
    WS_ATTN, WS_ATTN_QUANTIZED, WS_ATTN_TILED, WS_FORWARD, WS_PREDICT, WS_QUANTIZE,
)
