"""Thin ctypes binding of libvattn.so: argument marshalling only.

Every step of the path (memory mapping, KV append, prefill and decode attention) runs inside the
library; nothing here computes.  The function names match the C ABI declared in include/vattn.h.
If the shared library has not been built the import fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvattn.so")

POLICY_SYNC_UNMAP = 0
POLICY_DEFERRED = 1
FLAG_BACKGROUND = 0x10
FLAG_STATIC_BACKING = 0x20
FLAG_TENSOR_SLICING = 0x40


class VattnError(RuntimeError):
    pass


class _Config(ctypes.Structure):
    _fields_ = [("num_layers", ctypes.c_int32), ("max_batch", ctypes.c_int32), ("max_ctx", ctypes.c_int64),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("elem_bytes", ctypes.c_int32), ("page_group_bytes", ctypes.c_int64),
                ("phys_budget_bytes", ctypes.c_int64), ("device", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("lookahead_tokens", ctypes.c_int32), ("eager_page_groups", ctypes.c_int32),
                ("reclaim_threshold_page_groups", ctypes.c_int64)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2405_04437_amd/build.py` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    # host index arrays (int32 / int64) are passed as addresses, see _host_array
    vp, i32p, i64p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    dp = ctypes.POINTER(ctypes.c_double)
    lib.vattn_last_error.restype = ctypes.c_char_p
    lib.vattn_init.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(vp)]
    lib.vattn_destroy.argtypes = [vp]
    lib.vattn_alloc_reqid.argtypes = [vp]
    lib.vattn_free_reqid.argtypes = [vp, ctypes.c_int]
    lib.vattn_step.argtypes = [vp, i64p, ctypes.c_int]
    lib.vattn_kv_ptr.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.vattn_kv_ptr.restype = vp
    lib.vattn_query.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int), i64p, i64p]
    lib.vattn_stats.argtypes = [vp, i64p, i64p, i64p, i64p]
    lib.vattn_counters.argtypes = [vp, i64p, i64p, dp, dp]
    lib.vattn_append_kv.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32p, i32p, i64p, ctypes.c_int]
    lib.vattn_attn_prefill.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32p, i32p, i64p, ctypes.c_int, ctypes.c_float]
    lib.vattn_decode_workspace_bytes.argtypes = [vp, i64p, ctypes.c_int]
    lib.vattn_decode_workspace_bytes.restype = ctypes.c_int64
    lib.vattn_attn_decode.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32p, i64p, ctypes.c_int, ctypes.c_float, vp,
                                      ctypes.c_size_t]
    lib.vattn_attn_decode_static.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32p, i64p, ctypes.c_int, ctypes.c_float]
    lib.vattn_attn_decode_append.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, i32p, i64p, ctypes.c_int, ctypes.c_float, vp,
                                             ctypes.c_size_t]
    lib.vattn_attn_prefill_append.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, i32p, i32p, i64p, ctypes.c_int, ctypes.c_float]
    lib.vattn_attn_decode_paged.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, i32p, ctypes.c_int, i64p,
                                            ctypes.c_int, ctypes.c_float, vp, ctypes.c_size_t]
    lib.vattn_attn_prefill_paged.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int, i32p, ctypes.c_int, i32p, i64p,
                                             ctypes.c_int, ctypes.c_float]
    lib.vattn_set_timing.argtypes = [vp, ctypes.c_int]
    lib.vattn_kernel_time.argtypes = [vp, ctypes.c_int, dp, i64p]
    lib.vattn_set_decode_chunk.argtypes = [vp, ctypes.c_int]
    lib.vattn_set_decode_tuning.argtypes = [vp, ctypes.c_int]
    lib.vattn_set_decode_xcd_weights.argtypes = [vp, ctypes.c_void_p]
    lib.vattn_step_counters.argtypes = [vp, i64p, i64p, dp, dp, dp]
    lib.vattn_sync.argtypes = [vp]
    lib.vattn_vmm_microbench.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, dp]
    lib.vattn_mfma_microbench.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, dp]
    lib.vattn_stream_microbench.argtypes = [ctypes.c_int, ctypes.c_int64, dp]
    for name in ("vattn_init", "vattn_destroy", "vattn_alloc_reqid", "vattn_free_reqid", "vattn_step", "vattn_query",
                 "vattn_stats", "vattn_counters", "vattn_append_kv", "vattn_attn_prefill", "vattn_attn_decode",
                 "vattn_set_timing", "vattn_kernel_time", "vattn_set_decode_chunk", "vattn_set_decode_tuning",
                 "vattn_step_counters", "vattn_sync", "vattn_vmm_microbench", "vattn_attn_decode_paged", "vattn_attn_decode_append", "vattn_attn_prefill_paged",
                 "vattn_attn_prefill_append", "vattn_set_decode_xcd_weights",
                 "vattn_mfma_microbench", "vattn_stream_microbench", "vattn_attn_decode_static"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


lib = _load()

EXPORTED = ["vattn_init", "vattn_destroy", "vattn_alloc_reqid", "vattn_free_reqid", "vattn_step", "vattn_kv_ptr",
            "vattn_query", "vattn_stats", "vattn_counters", "vattn_append_kv", "vattn_attn_prefill",
            "vattn_decode_workspace_bytes", "vattn_attn_decode", "vattn_set_timing", "vattn_kernel_time",
            "vattn_set_decode_chunk", "vattn_set_decode_tuning", "vattn_step_counters",
            "vattn_sync", "vattn_vmm_microbench", "vattn_attn_decode_paged", "vattn_attn_decode_append", "vattn_attn_prefill_paged",
            "vattn_attn_prefill_append", "vattn_set_decode_xcd_weights",
            "vattn_mfma_microbench", "vattn_stream_microbench", "vattn_attn_decode_static", "vattn_last_error"]


def last_error() -> str:
    return (lib.vattn_last_error() or b"").decode()


def _host_array(a, dtype):
    """(array kept alive by the caller, its address): host index arrays are passed as plain addresses; an
    array that already has the right type and layout is used as it is (these calls sit on the critical
    path of a serving loop, between two GPU iterations)."""
    if type(a) is not np.ndarray or a.dtype != dtype or not a.flags.c_contiguous:
        a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.__array_interface__["data"][0]


def _i32(a: Sequence[int]):
    return _host_array(a, np.int32)


def _i64(a: Sequence[int]):
    return _host_array(a, np.int64)


def _ptr(x) -> int:
    """Device address of a torch tensor, or an int passed through."""
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


class Vattn:
    """One library context; method names mirror the C entry points without the prefix."""

    def __init__(self, num_layers: int, max_batch: int, max_ctx: int, num_q_heads: int, num_kv_heads: int,
                 head_dim: int, phys_budget_bytes: int, page_group_bytes: int = 0, elem_bytes: int = 2,
                 device: int = 0, policy: int = POLICY_SYNC_UNMAP, flags: int = 0, lookahead_tokens: int = 0,
                 eager_page_groups: int = 0, reclaim_threshold_page_groups: int = 0) -> None:
        cfg = _Config(num_layers, max_batch, max_ctx, num_q_heads, num_kv_heads, head_dim, elem_bytes,
                      page_group_bytes, phys_budget_bytes, device, policy | flags, lookahead_tokens,
                      eager_page_groups, reclaim_threshold_page_groups)
        h = ctypes.c_void_p()
        if lib.vattn_init(ctypes.byref(cfg), ctypes.byref(h)) != 0:
            raise VattnError("vattn_init: " + last_error())
        self._h = h
        self.max_batch = max_batch
        self.num_q_heads, self.num_kv_heads, self.head_dim = num_q_heads, num_kv_heads, head_dim

    def destroy(self) -> None:
        if self._h:
            lib.vattn_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- Table 4 of the paper --------------------------------------------------------------
    def alloc_reqid(self) -> int:
        return lib.vattn_alloc_reqid(self._h)

    def free_reqid(self, reqid: int) -> int:
        return lib.vattn_free_reqid(self._h, reqid)

    def step(self, seq_lens: Sequence[int]) -> int:
        arr, p = _i64(seq_lens)
        return lib.vattn_step(self._h, p, len(arr))

    # ---- introspection ---------------------------------------------------------------------
    def kv_ptr(self, layer: int, which: int, reqid: int) -> int:
        return lib.vattn_kv_ptr(self._h, layer, which, reqid) or 0

    def query(self, reqid: int) -> Tuple[int, int, int]:
        a, m, o = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
        if lib.vattn_query(self._h, reqid, ctypes.byref(a), ctypes.byref(m), ctypes.byref(o)) != 0:
            raise VattnError(last_error())
        return a.value, m.value, o.value

    def stats(self) -> Tuple[int, int, int, int]:
        v = [ctypes.c_int64() for _ in range(4)]
        lib.vattn_stats(self._h, *[ctypes.byref(x) for x in v])
        return tuple(x.value for x in v)

    def counters(self) -> Tuple[int, int, float, float]:
        a, b, c, d = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_double(), ctypes.c_double()
        lib.vattn_counters(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d))
        return a.value, b.value, c.value, d.value

    def step_counters(self) -> Tuple[int, int, float, float, float]:
        """(map calls inside step(), map calls by background passes, us in step(), us in passes, us waiting)."""
        a, b = ctypes.c_int64(), ctypes.c_int64()
        c, d, e = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        lib.vattn_step_counters(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d), ctypes.byref(e))
        return a.value, b.value, c.value, d.value, e.value

    def sync(self) -> int:
        return lib.vattn_sync(self._h)

    # ---- attention path --------------------------------------------------------------------
    def append_kv(self, layer: int, stream: int, k_new, v_new, reqids, cu_q, kv_len_before) -> int:
        r, rp = _i32(reqids)
        c, cp = _i32(cu_q)
        b, bp = _i64(kv_len_before)
        return lib.vattn_append_kv(self._h, layer, stream, _ptr(k_new), _ptr(v_new), rp, cp, bp, len(r))

    def attn_prefill(self, layer: int, stream: int, q, o, reqids, cu_q, kv_lens, scale: float) -> int:
        r, rp = _i32(reqids)
        c, cp = _i32(cu_q)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_prefill(self._h, layer, stream, _ptr(q), _ptr(o), rp, cp, kp, len(r), scale)

    def decode_workspace_bytes(self, kv_lens) -> int:
        k, kp = _i64(kv_lens)
        return lib.vattn_decode_workspace_bytes(self._h, kp, len(k))

    def attn_decode(self, layer: int, stream: int, q, o, reqids, kv_lens, scale: float, workspace,
                    workspace_bytes: int) -> int:
        r, rp = _i32(reqids)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_decode(self._h, layer, stream, _ptr(q), _ptr(o), rp, kp, len(r), scale,
                                     _ptr(workspace), workspace_bytes)

    def attn_decode_static(self, layer: int, stream: int, q, o, reqids, kv_lens, scale: float) -> int:
        r, rp = _i32(reqids)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_decode_static(self._h, layer, stream, _ptr(q), _ptr(o), rp, kp, len(r), scale)

    def attn_decode_append(self, layer: int, stream: int, q, k_new, v_new, o, reqids, kv_lens, scale: float, workspace,
                           workspace_bytes: int) -> int:
        r, rp = _i32(reqids)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_decode_append(self._h, layer, stream, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(o), rp, kp,
                                            len(r), scale, _ptr(workspace), workspace_bytes)

    def attn_prefill_append(self, layer: int, stream: int, q, k_new, v_new, o, reqids, cu_q, kv_lens, scale: float) -> int:
        r, rp = _i32(reqids)
        c, cp = _i32(cu_q)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_prefill_append(self._h, layer, stream, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(o), rp, cp, kp,
                                             len(r), scale)

    def attn_decode_paged(self, stream: int, q, o, k_pool, v_pool, num_blocks: int, block_tokens: int, block_table,
                          kv_lens, scale: float, workspace, workspace_bytes: int) -> int:
        t = np.ascontiguousarray(block_table, dtype=np.int32)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_decode_paged(self._h, stream, _ptr(q), _ptr(o), _ptr(k_pool), _ptr(v_pool), num_blocks,
                                           block_tokens, t.ctypes.data, t.shape[1],
                                           kp, len(k), scale, _ptr(workspace), workspace_bytes)

    def attn_prefill_paged(self, stream: int, q, o, k_pool, v_pool, num_blocks: int, block_tokens: int, block_table,
                           cu_q, kv_lens, scale: float) -> int:
        t = np.ascontiguousarray(block_table, dtype=np.int32)
        c, cp = _i32(cu_q)
        k, kp = _i64(kv_lens)
        return lib.vattn_attn_prefill_paged(self._h, stream, _ptr(q), _ptr(o), _ptr(k_pool), _ptr(v_pool), num_blocks,
                                            block_tokens, t.ctypes.data, t.shape[1], cp, kp, len(k), scale)

    # ---- measurement -----------------------------------------------------------------------
    def set_timing(self, enabled: bool) -> int:
        return lib.vattn_set_timing(self._h, 1 if enabled else 0)

    def kernel_time(self, which: int) -> Tuple[float, int]:
        t, n = ctypes.c_double(), ctypes.c_int64()
        if lib.vattn_kernel_time(self._h, which, ctypes.byref(t), ctypes.byref(n)) != 0:
            raise VattnError(last_error())
        return t.value, n.value

    def set_decode_chunk(self, tokens: int) -> int:
        return lib.vattn_set_decode_chunk(self._h, tokens)

    def set_decode_tuning(self, segments_per_slot: int) -> int:
        return lib.vattn_set_decode_tuning(self._h, segments_per_slot)

    def set_decode_xcd_weights(self, weights=None) -> int:
        if weights is None:
            return lib.vattn_set_decode_xcd_weights(self._h, None)
        w = np.ascontiguousarray(weights, dtype=np.float32)
        if w.shape != (8,):
            raise ValueError("eight weights, one per XCD")
        return lib.vattn_set_decode_xcd_weights(self._h, w.ctypes.data)


def vmm_microbench(page_group_bytes: int, count: int, device: int = 0):
    """Average microseconds per HIP virtual-memory call at one page-group size, then three mapping counts (see vattn_bench.h)."""
    out = (ctypes.c_double * 12)()
    if lib.vattn_vmm_microbench(device, page_group_bytes, count, out) != 0:
        raise VattnError("vattn_vmm_microbench: " + last_error())
    return list(out)


def mfma_microbench(normal_operands, rounds: int = 100000, device: int = 0, lds_operand: bool = False,
                    fma3: bool = False, exp2: bool = False):
    """(dense bf16 TFLOP/s, shader clock MHz) of a register-only MFMA loop on every CU, optionally with side work per
    matrix instruction: an operand read from LDS, three fp32 multiply-adds, one exp2 (see vattn_bench.h)."""
    out = (ctypes.c_double * 2)()
    mode = (1 if normal_operands else 0) | (2 if lds_operand else 0) | (4 if fma3 else 0) | (8 if exp2 else 0)
    if lib.vattn_mfma_microbench(device, mode, rounds, out) != 0:
        raise VattnError("vattn_mfma_microbench: " + last_error())
    return out[0], out[1]


def stream_microbench(nbytes: int = 4 << 30, device: int = 0) -> float:
    """GB/s of a kernel that only reads `nbytes` from HBM in the decode kernel's launch shape (see vattn.h)."""
    out = (ctypes.c_double * 1)()
    if lib.vattn_stream_microbench(device, nbytes, out) != 0:
        raise VattnError("vattn_stream_microbench: " + last_error())
    return out[0]
