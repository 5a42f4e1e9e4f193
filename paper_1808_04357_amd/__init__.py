"""MI355X-native Residual Gradient Compression hot path (RedSync, arXiv 1808.04357).

The package is a thin ctypes binding over ``librgc.so`` (hand-written HIP for gfx950, C ABI in
``include/rgc.h``).  It only marshals arguments: every step of the path runs in the library's
kernels.  PyTorch-ROCm tensors are used for device memory and streams.  There is no CPU
fallback: if the library is missing, importing the binding's entry points raises.
"""
from .binding import (  # noqa: F401
    RGC_ADD_TO_DST, RGC_NESTEROV, RGC_NO_HINTS, RGC_NO_MOMENTUM_MASK, RGC_ONE_VALUE, RGC_OVERWRITE,
    RGC_SELECT_LARGEST, RGC_SELECT_SMALLEST, RGC_STATUS_INDEX_ORDER, RGC_STATUS_INDEX_RANGE,
    RGC_THRESHOLD_SEARCH, RGC_VALIDATE, Context, LayerList, MessageList, RgcError, library_path,
    load_library, rgc_clip_coefficient, rgc_compress_layers, rgc_compress_layers_scaled,
    rgc_compress_layers_threshold, rgc_decompress_accumulate, rgc_k_for_density, rgc_message_means, rgc_message_means_noalloc, rgc_stream_yardstick,
    RGC_NOALLOC_MAX_LAYERS,
)
