"""ctypes front end of the C attention oracle (oracle/attention.c).

TEST INFRASTRUCTURE ONLY - see the header of attention.c.  The arithmetic lives in the C file; this
module compiles it with gcc, loads it and marshals numpy arrays.  Parity status: pinned (closed
forms, brute force in pure Python, a library SDPA special case, softmax row sums, chunking
invariance - see tests/test_oracle_attention.py).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention.c")
_LIB = os.path.join(_HERE, "_build", "liboracle_attention.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile attention.c into oracle/_build/liboracle_attention.so (gcc, OpenMP)."""
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_softmax_row.restype = ctypes.c_double
        lib.oracle_softmax_row.argtypes = [u16p, u16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_double, dp]
        lib.oracle_attention_request.restype = ctypes.c_int
        lib.oracle_attention_request.argtypes = [u16p, u16p, u16p, ctypes.c_int64, ctypes.c_int64,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_double, ctypes.POINTER(ctypes.c_int32),
                                                 ctypes.c_int64, dp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def softmax_row(q: np.ndarray, k: np.ndarray, kvh: int, scale: float) -> np.ndarray:
    """Softmax probabilities of one query vector q[D] against keys k[n, H, D], KV head kvh."""
    n, H, D = k.shape
    p = np.empty(n, dtype=np.float64)
    _load().oracle_softmax_row(_u16(q), _u16(k), n, H, D, kvh, float(scale),
                               p.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return p


def attention_request(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
                      rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Causal GQA attention of one request.

    q [q_len, Hq, D], k/v [kv_len, H, D] as bf16 bit patterns (uint16).  Returns float64
    [len(rows) or q_len, Hq, D].  Query row i sees keys 0 .. kv_len - q_len + i.
    """
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    q_len, Hq, D = q.shape
    kv_len, H, Dk = k.shape
    assert Dk == D and v.shape == k.shape
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        n_rows = len(rows)
        rp = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    else:
        n_rows = q_len
        rp = None
    out = np.empty((n_rows, Hq, D), dtype=np.float64)
    rc = _load().oracle_attention_request(_u16(q), _u16(k), _u16(v), q_len, kv_len, Hq, H, D,
                                          float(scale), rp, n_rows,
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError("oracle_attention_request rejected its arguments")
    return out


def attention_batch(q: np.ndarray, cu_q: Sequence[int], ks: List[np.ndarray], vs: List[np.ndarray],
                    scale: float) -> np.ndarray:
    """Attention evaluated request by request, as Eq. 2 is meant for a batch: q is packed
    [sum q_len, Hq, D] with prefix sums cu_q; returns float64 of the same shape."""
    out = np.empty(q.shape, dtype=np.float64)
    for r in range(len(ks)):
        a, b = int(cu_q[r]), int(cu_q[r + 1])
        if b > a:
            out[a:b] = attention_request(q[a:b], ks[r], vs[r], scale)
    return out
