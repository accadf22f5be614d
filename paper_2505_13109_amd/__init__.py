"""MI355X-native FreeKV retrieval-decode path: a thin ctypes binding over libfreekv.so.

All arithmetic of the path runs in the HIP kernels of the library; this package only
marshals arguments (PyTorch supplies device memory and streams).  There is no CPU
fallback: importing works without a GPU (so the symbols can be checked), creating a
context does not.
"""
from .binding import (  # noqa: F401
    FKV_DTYPE_FP16, FKV_DTYPE_BF16, FKV_PLACE_HBM, FKV_PLACE_HOST,
    FKV_USE_ACTIVE, FKV_USE_PENDING, FKV_USE_BY_FLAG,
    FKV_HEADS_ALL, FKV_HEADS_FLAGGED, FKV_HEADS_UNFLAGGED, FKV_RECALL_GATHER, FKV_RECALL_MEMCPY,
    FkvConfig, FreeKV, FreeKVError, lib, lib_path, EXPORTED_SYMBOLS,
)
