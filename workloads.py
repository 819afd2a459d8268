"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This module only *draws inputs*: request-length mixes, N(0,1) tensors rounded to bf16, and the
model shapes of the paper's table of evaluated models and hardware (Table 5:
Yi-6B 32/4 heads, Llama-3-8B 32/8, Yi-34B 56/8; head dimension 128).  It contains none of the
method's arithmetic (no attention, no page counting) so that the HIP path and the oracle can both
be fed from it without sharing any computation.

The synthetic tensors stand in for the paper's arXiv-Summarization / OpenChat traces and the model
weights, none of which are available offline: only shapes and context-length ranges are kept.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 20240507


@dataclass(frozen=True)
class Shape:
    """Attention shape of one worker: query heads, KV heads (H), head dim (D), bytes/elem (P)."""

    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    num_layers: int
    elem_bytes: int = 2

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def token_bytes(self) -> int:
        """Bytes one token occupies in one K (or V) buffer of one layer: H*D*P."""
        return self.num_kv_heads * self.head_dim * self.elem_bytes


TINY = Shape("tiny", 8, 2, 64, 2)
YI_6B = Shape("yi-6b", 32, 4, 128, 32)
LLAMA3_8B = Shape("llama-3-8b", 32, 8, 128, 32)
YI_34B = Shape("yi-34b", 56, 8, 128, 60)


@dataclass
class Workload:
    """One named configuration: a shape plus per-request (q_len, kv_len) pairs.

    kv_len counts the tokens visible to the *last* query row of the request, i.e. the context
    after the new q_len tokens were appended.  Decode requests have q_len == 1.
    """

    name: str
    shape: Shape
    seed: int
    q_lens: List[int]
    kv_lens: List[int]
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return len(self.q_lens)


def _rng(cfg_index: int) -> np.random.Generator:
    return np.random.default_rng(SEED_BASE + cfg_index)


def _uniform_lengths(rng: np.random.Generator, lo: int, hi: int, n: int) -> List[int]:
    return [int(x) for x in rng.integers(lo, hi, size=n, endpoint=True)]


def config(index: int) -> Workload:
    """The five benchmark configurations, index 0..4, lengths drawn from the config's own seed."""
    rng = _rng(index)
    if index == 0:
        kv = _uniform_lengths(rng, 1, 512, 4)
        return Workload("C1-tiny-decode", TINY, SEED_BASE, [1] * 4, kv, "batch 4, ctx U[1,512]")
    if index == 1:
        kv = _uniform_lengths(rng, 1024, 16384, 64)
        return Workload("C2-yi6b-decode", YI_6B, SEED_BASE + 1, [1] * 64, kv, "batch 64, ctx U[1024,16384]")
    if index == 2:
        ql = _uniform_lengths(rng, 4096, 32768, 8)
        return Workload("C3-llama3-8b-prefill", LLAMA3_8B, SEED_BASE + 2, ql, list(ql), "8 prompts U[4096,32768]")
    if index == 3:
        kv = _uniform_lengths(rng, 2048, 32768, 128)
        w = Workload(
            "C4-yi34b-mixed", YI_34B, SEED_BASE + 3, [1] * 128 + [2048], kv + [8192 + 2048],
            "128 decodes ctx U[2048,32768] + one 2048-token chunk appended at 8192; 10% reqId churn/step",
        )
        w.extra["churn_fraction"] = 0.10
        w.extra["ctx_range"] = (2048, 32768)
        return w
    if index == 4:
        w = Workload("C5-llama3-8b-long", LLAMA3_8B, SEED_BASE + 4, [131072], [131072],
                     "131072-token prefill, then 256 decode steps")
        w.extra["decode_steps"] = 256
        return w
    raise IndexError(index)


# ---------------------------------------------------------------------------------------------
# bf16 helpers (storage format only: round-to-nearest-even narrowing, exact widening)
# ---------------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest-even) and return the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape: Tuple[int, ...]) -> np.ndarray:
    """i.i.d. N(0,1) samples rounded to bf16, returned as uint16 bit patterns."""
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


@dataclass
class AttnInputs:
    """Host-side tensors of one attention call (bf16 bit patterns).

    q:  [sum(q_lens), Hq, D]  packed over requests in order
    k, v: one array per request, [kv_len, H, D] (token-major, as the KV cache stores it)
    """

    q: np.ndarray
    k: List[np.ndarray]
    v: List[np.ndarray]
    cu_q: np.ndarray  # int32 [n+1] prefix sums of q_lens


def draw_attention_inputs(shape: Shape, q_lens: List[int], kv_lens: List[int], seed: int) -> AttnInputs:
    rng = np.random.default_rng(seed)
    cu = np.zeros(len(q_lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(q_lens)
    q = normal_bf16(rng, (int(cu[-1]), shape.num_q_heads, shape.head_dim))
    k = [normal_bf16(rng, (int(L), shape.num_kv_heads, shape.head_dim)) for L in kv_lens]
    v = [normal_bf16(rng, (int(L), shape.num_kv_heads, shape.head_dim)) for L in kv_lens]
    return AttnInputs(q, k, v, cu)


def softmax_scale(head_dim: int) -> float:
    return 1.0 / float(np.sqrt(head_dim))


def sample_rows(q_len: int, count: int, seed: int, boundaries: Optional[List[int]] = None) -> np.ndarray:
    """A seeded sample of query-row indices in [0, q_len): always row 0 and the last row, rows next
    to the given boundaries (tile or page edges), and uniformly drawn rows for the rest."""
    rows = {0, q_len - 1}
    for b in boundaries or []:
        for d in (-1, 0, 1):
            if 0 <= b + d < q_len:
                rows.add(b + d)
    rng = np.random.default_rng(seed)
    while len(rows) < min(count, q_len):
        rows.add(int(rng.integers(0, q_len)))
    return np.array(sorted(rows), dtype=np.int32)


# ---------------------------------------------------------------------------------------------
# Serving-loop traces for the allocator (arrivals / completions), in the shape of Algorithm 1
# ---------------------------------------------------------------------------------------------

@dataclass
class TraceEvent:
    kind: str            # "alloc" | "free" | "step"
    slot: int = -1       # framework-side request handle the event refers to (alloc/free)
    prompt_len: int = 0  # for alloc
    seq_lens: Optional[List[int]] = None  # for step, filled by the driver of the trace


def serving_trace(seed: int, max_batch: int, iterations: int, prompt_range: Tuple[int, int],
                  out_range: Tuple[int, int], arrival_p: float = 0.5) -> List[Tuple[str, int, int]]:
    """A seeded list of framework-level events: ("arrive", prompt_len, out_len) or ("iterate",0,0).

    The consumer runs Algorithm 1 of the paper over it: admitted requests get a reqId and their
    prompt length, every iteration calls step(), finished requests are freed, the others grow by
    one token.  This function only draws the numbers.
    """
    rng = np.random.default_rng(seed)
    ev: List[Tuple[str, int, int]] = []
    for _ in range(iterations):
        n_arrive = int(rng.binomial(max(1, max_batch // 4), arrival_p))
        for _ in range(n_arrive):
            ev.append(("arrive", int(rng.integers(prompt_range[0], prompt_range[1], endpoint=True)),
                       int(rng.integers(out_range[0], out_range[1], endpoint=True))))
        ev.append(("iterate", 0, 0))
    return ev
