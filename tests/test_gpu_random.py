"""Seeded random shapes through every attention entry point against the CPU oracle: head counts, head
dimension, batch size, chunk lengths (empty, single-token, inside and across tiles) and the position a chunk
is appended at are drawn per case; prefill and decode, each plain and with the KV append fused in."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from parity import check

pytestmark = pytest.mark.gpu
MiB = 1024 * 1024


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128]))
    H = int(rng.choice([1, 2, 3, 4, 8]))
    g = int(rng.choice([1, 2, 4, 5, 7, 8, 17]))
    n = int(rng.integers(1, 10))
    kinds = rng.integers(0, 6, size=n)
    q_lens = [int({0: 0, 1: 1, 2: rng.integers(2, 64), 3: rng.integers(64, 400), 4: rng.integers(400, 900), 5: 64 * rng.integers(1, 6)}[int(k)]) for k in kinds]
    offs = [int(rng.choice([0, 0, 1, 63, 64, 65, rng.integers(0, 700)])) for _ in range(n)]
    if sum(q_lens) == 0:
        q_lens[0] = 5
    kv_lens = [max(1, q + o) for q, o in zip(q_lens, offs)]      # a request with no query rows still has a context
    return W.Shape(f"r{seed}", H * g, H, D, 1), q_lens, kv_lens


@pytest.mark.parametrize("seed", range(48))
def test_random_shapes_all_entry_points(seed):
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession, bits_to_tensor, tensor_to_f32

    shape, q_lens, kv_lens = _case(seed)
    n, H, D = len(q_lens), shape.num_kv_heads, shape.head_dim
    offs = [k - q for k, q in zip(kv_lens, q_lens)]
    scale = W.softmax_scale(D)
    G = int(np.random.default_rng(seed).choice([4096, 64 * 1024, 2 * MiB]))
    per_req = (max(kv_lens) * shape.token_bytes + G - 1) // G * G
    tag = f"seed {seed}: Hq={shape.num_q_heads} H={H} D={D} q={q_lens} kv={kv_lens} G={G}"

    # prefill: plain over a fully written cache, then fused with the chunk rows poisoned beforehand
    inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed)
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    s = KvSession(shape.num_q_heads, H, D, n + 1, max(kv_lens), per_req * 2 * (n + 1), 1, G)
    ids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    check(tensor_to_f32(s.prefill(0, q, ids, inp.cu_q, kv_lens, scale)), want, "prefill, " + tag)
    poison = torch.full((int(inp.cu_q[-1]), H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    s.append(0, poison, poison, ids, inp.cu_q, offs)
    k_new = bits_to_tensor(np.concatenate([k[o:] for k, o in zip(inp.k, offs)]))
    v_new = bits_to_tensor(np.concatenate([v[o:] for v, o in zip(inp.v, offs)]))
    o = torch.empty_like(q)
    assert s.va.attn_prefill_append(0, s.stream, q, k_new, v_new, o, ids, inp.cu_q, kv_lens, scale) == 0, P.last_error()
    check(tensor_to_f32(o), want, "fused prefill, " + tag)
    s.close()

    # decode over the same contexts: plain, then fused with the newest token poisoned beforehand
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed + 100)
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    s = KvSession(shape.num_q_heads, H, D, n + 1, max(kv_lens), per_req * 2 * (n + 1), 1, G)
    ids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    check(tensor_to_f32(s.decode(0, q, ids, kv_lens, scale)), want, "decode, " + tag)
    poison = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    s.append(0, poison, poison, ids, np.arange(n + 1), [L - 1 for L in kv_lens])
    k_new = bits_to_tensor(np.stack([k[-1] for k in inp.k]))
    v_new = bits_to_tensor(np.stack([v[-1] for v in inp.v]))
    o = torch.empty_like(q)
    ws = s.workspace(kv_lens)
    assert s.va.attn_decode_append(0, s.stream, q, k_new, v_new, o, ids, kv_lens, scale, ws, ws.numel()) == 0, P.last_error()
    check(tensor_to_f32(o), want, "fused decode, " + tag)
    s.close()
