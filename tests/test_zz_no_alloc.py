"""The allocation-free decode entry point (vattn_attn_decode_static: split-K partials in a device array the
library owns) against vattn_attn_decode with a caller-owned workspace, through the C ABI: two calls in a
row on the same GPU array, the second with a smaller batch, then the size limits.  Both entry points run
the same kernels over the same plan, so the outputs must agree bit for bit; the oracle check on top holds
the pair to the attention tolerance."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from parity import check

pytestmark = pytest.mark.gpu
MiB = 1024 * 1024


def _session(shape, n, max_ctx, G=2 * MiB):
    from paper_2405_04437_amd.runtime import KvSession

    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    return KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + 2, max_ctx, per_req * 2 * (n + 2), 1, G)


def test_static_scratch_decode_equals_workspace_decode_on_two_calls_in_a_row():
    import torch
    from paper_2405_04437_amd import last_error
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_bits, tensor_to_f32

    shape = W.Shape("t", 32, 4, 128, 1)
    scale = W.softmax_scale(shape.head_dim)
    # first call: 24 requests, ragged, several split-K segments per request and several requests per segment
    kv_big = [1, 31, 32, 33, 700, 4096, 4097, 9000, 12345, 2, 640, 641] * 2
    # second call: a smaller batch (a subset of the requests, shorter contexts) - stale partials of the first
    # call stay in the array and must not be read
    sub = [0, 4, 7, 8, 13, 20]
    inp = W.draw_attention_inputs(shape, [1] * len(kv_big), kv_big, seed=77)
    s = _session(shape, len(kv_big), max(kv_big))
    ids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    for which, (slots, lens) in enumerate([(list(range(len(kv_big))), kv_big), (sub, [max(1, kv_big[i] // 2) for i in sub])]):
        print(f"static decode call {which}: {len(slots)} requests", flush=True)
        qs = q[torch.tensor(slots, device="cuda")].contiguous()
        rid = [ids[i] for i in slots]
        want_gpu = s.decode(0, qs, rid, lens, scale)
        got = torch.full_like(qs, float("nan"))
        rc = s.va.attn_decode_static(0, s.stream, qs, got, rid, lens, scale)
        assert rc == 0, last_error()
        torch.cuda.synchronize()
        assert np.array_equal(tensor_to_bits(got), tensor_to_bits(want_gpu)), f"call {which}: static and workspace variants differ"
        ks = [inp.k[i][:L] for i, L in zip(slots, lens)]
        vs = [inp.v[i][:L] for i, L in zip(slots, lens)]
        want = OA.attention_batch(tensor_to_bits(qs), np.arange(len(slots) + 1), ks, vs, scale)
        check(tensor_to_f32(got), want, f"static decode call {which}")
    s.close()


def test_static_scratch_decode_refuses_what_does_not_fit():
    import torch
    from paper_2405_04437_amd import last_error
    from paper_2405_04437_amd.runtime import KvSession

    # more than 256 requests: the index arrays would need the staging ring
    shape = W.Shape("t", 8, 2, 64, 1)
    n = 257
    G = 64 * 1024
    s = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n, 64, 2 * n * G, 1, G)
    ids = [s.admit(8) for _ in range(n)]
    s.step()
    q = torch.zeros((n, 8, 64), device="cuda", dtype=torch.bfloat16)
    o = torch.empty_like(q)
    assert s.va.attn_decode_static(0, s.stream, q, o, ids, [8] * n, 0.125) == -1 and "at most 256" in last_error()
    assert s.va.attn_decode_static(0, s.stream, q, o, ids[:256], [8] * 256, 0.125) == 0, last_error()
    torch.cuda.synchronize()
    s.close()
    # partials larger than the library-owned array: 256 requests x 256 query heads need 42 MB
    s = KvSession(256, 2, 128, 256, 64, 2 * 256 * G, 1, G)
    ids = [s.admit(8) for _ in range(256)]
    s.step()
    q = torch.zeros((256, 256, 128), device="cuda", dtype=torch.bfloat16)
    o = torch.empty_like(q)
    assert s.va.attn_decode_static(0, s.stream, q, o, ids, [8] * 256, 0.1) == -1 and "library-owned array" in last_error()
    s.close()


def test_static_scratch_decode_replays_from_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (no allocation, no copy, no upload inside the call) and
    replayed several times with eager work and synchronisations between the replays; every replay must equal the eager
    vattn_attn_decode over the same, freshly drawn queries."""
    import torch
    from paper_2405_04437_amd import last_error
    from paper_2405_04437_amd.runtime import bits_to_tensor

    shape = W.Shape("t", 32, 4, 128, 1)
    scale = W.softmax_scale(shape.head_dim)
    kv = [700, 4097, 33, 9000]
    inp = W.draw_attention_inputs(shape, [1] * len(kv), kv, seed=5)
    s = _session(shape, len(kv), max(kv))
    ids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    o, o_ref = torch.empty_like(q), torch.empty_like(q)
    side = torch.cuda.Stream()
    assert s.va.attn_decode_static(0, side.cuda_stream, q, o, ids, kv, scale) == 0, last_error()   # first use, outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        assert s.va.attn_decode_static(0, torch.cuda.current_stream().cuda_stream, q, o, ids, kv, scale) == 0, last_error()
    for rep in range(4):
        q.copy_(bits_to_tensor(W.normal_bf16(np.random.default_rng(rep), tuple(q.shape))))        # eager work between the replays
        o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ws = s.workspace(kv)
        assert s.va.attn_decode(0, s.stream, q, o_ref, ids, kv, scale, ws, ws.numel()) == 0, last_error()
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), f"replay {rep} differs from the eager call"
    del graph
    s.close()
