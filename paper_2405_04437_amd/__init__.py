"""MI355X-native contiguous-KV attention with on-demand physical memory (vAttention's hot path).

The package is a thin binding over libvattn.so (HIP kernels + C ABI, sources in csrc/).  Importing it
requires the built library; see build.py.
"""
from .binding import (EXPORTED, FLAG_BACKGROUND, FLAG_STATIC_BACKING, FLAG_TENSOR_SLICING, LIB_PATH, POLICY_DEFERRED,
                      POLICY_SYNC_UNMAP, Vattn, VattnError, last_error, lib, mfma_microbench, stream_microbench, vmm_microbench)

__all__ = ["EXPORTED", "FLAG_BACKGROUND", "FLAG_STATIC_BACKING", "FLAG_TENSOR_SLICING", "vmm_microbench", "mfma_microbench", "stream_microbench", "LIB_PATH", "POLICY_DEFERRED", "POLICY_SYNC_UNMAP", "Vattn", "VattnError", "last_error", "lib"]
