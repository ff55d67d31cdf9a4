"""MI355X-native L2L (layer-to-layer) relay execution: the device library's Python binding and the
step driver above it."""
from .binding import (Context, EPS, L2LError, make_config, layer_layout, embed_layout, cls_layout, lib,  # noqa: F401
                      L2L_F32, L2L_BF16, L2L_FP16, L2L_OK, L2L_E_ARG, L2L_E_STATE, L2L_E_HIP, L2L_E_NOMEM, EXPORTS, LIB_PATH)
