"""MI355X-native multi-tenant inference worker runtime (HIP, gfx950) and its thin binding."""
from .binding import (Context, MtError, debug_big_tile_rows, debug_big_tile_walk, debug_conv_row_tiling, debug_copy, debug_mfma_rate, layer_spec, load_library, model_footprint, version,  # noqa: F401
                      MT_ACT_GELU, MT_ACT_NONE, MT_ACT_RELU, MT_ADD, MT_BF16, MT_CONV2D, MT_F32, MT_FC, MT_GAP, MT_MAXPOOL,
                      MT_MAX_LAYERS, mt_layer_spec)
from .torch_io import Served, context_for, register_tenants, serve  # noqa: F401
