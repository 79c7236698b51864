"""MI355X-native implementation of QTALE's inference hot path (token-adaptive, int4 weight-quantized
decoder-layer forward).  All compute lives in libqtale.so (HIP kernels behind a C ABI, include/qtale.h);
this package is the ctypes binding plus small device-memory helpers."""
from .binding import *  # noqa: F401,F403
from .binding import load_library, LIB_PATH, EXPORTS  # noqa: F401
from .layers import quantize_layer, cfg_from_shape  # noqa: F401
