"""MI355X-native TinyKG hot path: activation compressor + attentive KG aggregation.

The compute lives in libtinykg.so (hand-written HIP for gfx950, C ABI declared in
include/tinykg.h); this package is only its ctypes binding.
"""
from .binding import (ROUND_NEAREST, ROUND_STOCHASTIC, Graph, SavedContext, TinyKGError,  # noqa: F401
                      alloc_quantized, lib, tinykg_dequantize, tinykg_kg_aggregate_bwd,
                      tinykg_kg_aggregate_fwd, tinykg_kg_aggregate_workspace_bytes,
                      tinykg_num_groups, tinykg_packed_bytes, tinykg_profile_copy, tinykg_profile_enable,
                      tinykg_profile_report, tinykg_quantize)
