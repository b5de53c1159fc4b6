"""MI355X-native TinyKG hot path: activation compressor + attentive KG aggregation.

The compute lives in libtinykg.so (hand-written HIP for gfx950, C ABI declared in
include/tinykg.h); this package is only its ctypes binding.
"""
from .binding import (tinykg_bpr_grad, tinykg_bpr_loss, tinykg_gather_rows,  # noqa: F401
                      tinykg_scatter_add_rows, tinykg_fill_zero,
                      ROUND_NEAREST, ROUND_STOCHASTIC, Graph, SavedContext, TinyKGError,  # noqa: F401
                      alloc_quantized, lib, tinykg_dequantize, tinykg_kg_aggregate_bwd,
                      tinykg_kg_aggregate_fwd, tinykg_kg_aggregate_workspace_bytes,
                      tinykg_kg_uniform_bwd, tinykg_kg_uniform_fwd,
                      tinykg_num_groups, tinykg_packed_bytes, tinykg_profile_copy, tinykg_profile_enable,
                      tinykg_profile_report, tinykg_profile_select, tinykg_quantize, tinykg_quantize_bf16,
                      NormContext, tinykg_batchnorm_fwd, tinykg_batchnorm_bwd, tinykg_batchnorm_bwd_static, tinykg_readout_ids, tinykg_kg_max_fwd, tinykg_kg_max_bwd)
from .stack import KGStack  # noqa: F401,E402
