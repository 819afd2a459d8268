"""MI355X-native contiguous-KV attention with on-demand physical memory (vAttention's hot path).

The package is a thin binding over libvattn.so (HIP kernels + C ABI, sources in csrc/).  Importing it
requires the built library; see build.py.
"""
from .binding import (EXPORTED, LIB_PATH, POLICY_DEFERRED, POLICY_SYNC_UNMAP, Vattn, VattnError, last_error, lib)

__all__ = ["EXPORTED", "LIB_PATH", "POLICY_DEFERRED", "POLICY_SYNC_UNMAP", "Vattn", "VattnError", "last_error", "lib"]
