"""MI355X-native placement-aware MoE layer (one edge server's forward of the
Prism system, arXiv 2508.12851): HIP kernels behind the C ABI of
include/prism.h, plus a thin ctypes binding.  Importing this package does not
load the library; the first call (or load_library()) does."""
from .binding import (  # noqa: F401
    ExpertWeights, LayerDesc, LayerOut, PrismError, WeightTable, alloc_layer_out, alloc_workspace,
    load_library, make_desc, prism_combine, prism_dispatch, prism_expert_ffn, prism_moe_layer,
    prism_route, torch_dtype, workspace_bytes, LIB_PATH, SYMBOLS, STAGES,
    prism_ceiling_mfma_bf16, prism_ceiling_hbm_read, prism_pack_remote, prism_combine_remote,
    prism_debug_check_weights, prism_pack_weights, prism_layer_permutation, LayerPermutation,
    prism_moe_layer_static, STATIC_SCRATCH_BYTES, prism_ceiling_hbm_read_pattern,
)
