"""MI355X-native forward pass of binary-weight / binary-activation acoustic models (arXiv 1706.09453).

The product is the C-ABI library libbnn_hip.so (include/bnn.h); this package is its thin binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTED, LIB_PATH, BnnError, bnn_layer_desc, make_layer_array  # noqa: F401
