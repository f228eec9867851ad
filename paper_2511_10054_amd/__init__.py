"""BuddyMoE layer forward for MI355X (gfx950): thin binding over libbuddymoe.so.

Every step of the layer runs in the HIP library; this package only marshals
arguments (torch tensors -> device pointers).  There is no CPU fallback: if
the library has not been built, importing `binding` symbols raises.
"""
from .binding import (  # noqa: F401
    BM_BF16, BM_F32, BM_REMAP_UNIQUE, BM_RENORM_TOPK, BM_Y_F32,
    BM_GATE_TAE, BM_GATE_MARGIN, BM_REPLACE_BUDGET, BM_GATE_DIST, BM_PSI_TOKEN,
    LayerDesc, Weights, BuddyMoEError,
    bm_route_topk, bm_buddy_remap, bm_permute_by_expert, bm_moe_forward, bm_moe_forward_static,
    BM_STATIC_WORKSPACE_BYTES,
    bm_workspace_bytes, bm_validate_tables, bm_strerror, library_path, load_library,
    bm_packed_bytes, bm_pack_weights, bm_coactivation_accumulate, bm_build_buddy_table, bm_stream_read,
)
