"""MI355X-native K-FAC hot path: thin ctypes binding over the C ABI in include/kfac.h.

Argument marshalling only: every arithmetic step runs in the HIP kernels of
libkfac_hip.so.  There is no CPU fallback; load() raises when the library is missing.
"""
from .binding import (  # noqa: F401
    load, is_built, lib_path, Context, KfacError, make_layer, layer_struct,
    KFAC_OK, KFAC_ERR_INVALID_ARG, KFAC_ERR_NOT_SPD, KFAC_ERR_WORKSPACE, KFAC_ERR_DEVICE,
    EXPORTS, KERNEL_CLASSES, OPTIONS, place_inversions,
)
