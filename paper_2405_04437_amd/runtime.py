"""Convenience plumbing around the binding for tests, smoke() and bench.py: torch tensors for Q/O and
the decode workspace, the current torch stream, and bf16 bit-pattern <-> tensor conversion.  Holds no
arithmetic of the method - every numerical step happens in libvattn.so."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from .binding import POLICY_SYNC_UNMAP, Vattn, VattnError, last_error


def bits_to_tensor(bits: np.ndarray, device: str = "cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def tensor_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def tensor_to_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


class KvSession:
    """A library context plus the framework-side state of Algorithm 1 (cache_seq_len per reqId)."""

    def __init__(self, num_q_heads: int, num_kv_heads: int, head_dim: int, max_batch: int, max_ctx: int,
                 phys_budget_bytes: int, num_layers: int = 1, page_group_bytes: int = 0,
                 policy: int = POLICY_SYNC_UNMAP, device: int = 0, flags: int = 0, lookahead_tokens: int = 0,
                 eager_page_groups: int = 0, reclaim_threshold_page_groups: int = 0) -> None:
        if not torch.cuda.is_available():
            raise RuntimeError("KvSession needs a GPU: the HIP path has no CPU fallback")
        torch.cuda.set_device(device)
        self.va = Vattn(num_layers, max_batch, max_ctx, num_q_heads, num_kv_heads, head_dim, phys_budget_bytes,
                        page_group_bytes, 2, device, policy, flags, lookahead_tokens, eager_page_groups,
                        reclaim_threshold_page_groups)
        self.Hq, self.H, self.D = num_q_heads, num_kv_heads, head_dim
        self.B = max_batch
        self.num_layers = num_layers
        self.seq_lens = [0] * max_batch
        self._ws: Optional[torch.Tensor] = None

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream().cuda_stream

    def close(self) -> None:
        torch.cuda.synchronize()
        self.va.destroy()

    def _check(self, rc: int, what: str) -> None:
        if rc != 0:
            raise VattnError(f"{what}: {last_error()}")

    # ---- Algorithm 1 pieces ----------------------------------------------------------------
    def admit(self, prompt_len: int) -> int:
        r = self.va.alloc_reqid()
        if r < 0:
            raise VattnError("alloc_reqid: " + last_error())
        self.seq_lens[r] = prompt_len
        return r

    def finish(self, reqid: int) -> None:
        self.seq_lens[reqid] = 0
        self._check(self.va.free_reqid(reqid), "free_reqid")

    def step(self) -> None:
        self._check(self.va.step(self.seq_lens), "step")

    # ---- attention path --------------------------------------------------------------------
    def append(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, reqids: Sequence[int],
               cu_q: Sequence[int], kv_before: Sequence[int]) -> None:
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == torch.bfloat16
        self._check(self.va.append_kv(layer, self.stream, k_new, v_new, reqids, cu_q, kv_before), "append_kv")

    def prefill(self, layer: int, q: torch.Tensor, reqids, cu_q, kv_lens, scale: float,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        assert q.is_contiguous() and q.dtype == torch.bfloat16
        o = torch.empty_like(q) if out is None else out
        self._check(self.va.attn_prefill(layer, self.stream, q, o, reqids, cu_q, kv_lens, scale), "attn_prefill")
        return o

    def workspace(self, kv_lens) -> torch.Tensor:
        need = self.va.decode_workspace_bytes(kv_lens)
        if need < 0:
            raise VattnError("decode_workspace_bytes: " + last_error())
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    def decode(self, layer: int, q: torch.Tensor, reqids, kv_lens, scale: float,
               out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
        assert q.is_contiguous() and q.dtype == torch.bfloat16
        o = torch.empty_like(q) if out is None else out
        ws = self.workspace(kv_lens) if ws is None else ws
        self._check(self.va.attn_decode(layer, self.stream, q, o, reqids, kv_lens, scale, ws, ws.numel()),
                    "attn_decode")
        return o

    # ---- helpers for tests -----------------------------------------------------------------
    def load_contexts(self, ks: List[np.ndarray], vs: List[np.ndarray], layer: int = 0) -> List[int]:
        """Admit one request per (K, V) pair given as bf16 bit patterns [kv_len, H, D], back them with
        step() and write them through append_kv.  Returns the reqIds."""
        reqids = [self.admit(int(k.shape[0])) for k in ks]
        self.step()
        cu = np.zeros(len(ks) + 1, dtype=np.int64)
        cu[1:] = np.cumsum([k.shape[0] for k in ks])
        k_all = bits_to_tensor(np.concatenate(ks, axis=0))
        v_all = bits_to_tensor(np.concatenate(vs, axis=0))
        self.append(layer, k_all, v_all, reqids, cu, [0] * len(ks))
        return reqids
