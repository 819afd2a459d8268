"""GPU parity of the HIP attention path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from parity import check

pytestmark = pytest.mark.gpu
KiB, MiB = 1024, 1024 * 1024


def _session(shape, n, max_ctx, G=2 * MiB, layers=1, policy=0, slack=2):
    from paper_2405_04437_amd.runtime import KvSession

    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    budget = per_req * 2 * layers * (n + slack)
    return KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + slack, max_ctx, budget, layers, G, policy)


def _run_decode(shape, kv_lens, seed, G=2 * MiB, chunk=0):
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed)
    scale = W.softmax_scale(shape.head_dim)
    s = _session(shape, n, max(kv_lens), G)
    reqids = s.load_contexts(inp.k, inp.v)
    if chunk:
        assert s.va.set_decode_chunk(chunk) == 0
    got = tensor_to_f32(s.decode(0, bits_to_tensor(inp.q), reqids, kv_lens, scale))
    s.close()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    return got, want, inp


def test_config1_tiny_decode_matches_oracle():
    wl = W.config(0)
    got, want, _ = _run_decode(wl.shape, wl.kv_lens, wl.seed)
    check(got, want, "C1 decode")


@pytest.mark.parametrize("Hq,H,D", [(8, 2, 64), (32, 4, 128), (56, 8, 128), (4, 4, 128), (40, 2, 64), (7, 1, 128)])
def test_decode_shapes_ragged_lengths(Hq, H, D):
    shape = W.Shape("t", Hq, H, D, 1)
    kv_lens = [1, 2, 31, 32, 33, 63, 64, 65, 511, 512, 513, 1000, 2049]
    got, want, _ = _run_decode(shape, kv_lens, seed=Hq * 31 + D)
    check(got, want, f"decode Hq={Hq} H={H} D={D}")


@pytest.mark.parametrize("Hq,H,D", [(32, 4, 128), (8, 2, 64)])
def test_decode_batch_larger_than_the_inline_index_arrays(Hq, H, D):
    """More than 256 requests: reqIds, lengths and tile prefix sums no longer fit the kernel-argument segment and
    travel through the staging ring instead (append, split-K, both reduce kernels: short contexts take the
    one-wave reduce, the two long ones the general one)."""
    shape = W.Shape("t", Hq, H, D, 1)
    rng = np.random.default_rng(D)
    kv_lens = rng.integers(1, 200, size=298).tolist() + [5000, 7001]
    got, want, _ = _run_decode(shape, kv_lens, seed=3)
    check(got, want, f"decode with {len(kv_lens)} requests")
    got, want, _ = _run_decode(shape, kv_lens[:298], seed=4)
    check(got, want, "decode with 298 short requests")


@pytest.mark.parametrize("chunk", [32, 64, 256, 512, 4096])
def test_decode_invariant_to_chunk_size(chunk):
    shape = W.YI_6B
    kv_lens = [777, 3000, 1, 4097]
    got, want, _ = _run_decode(shape, kv_lens, seed=5, chunk=chunk)
    check(got, want, f"decode chunk={chunk}")


@pytest.mark.parametrize("weights", [None, [1] * 8, [4, 0.25, 1, 1, 0.25, 4, 2, 0.5], [0.25, 0.25, 0.25, 0.25, 0.25, 0.25, 0.25, 4]])
def test_decode_invariant_to_xcd_weights(weights):
    """Segment lengths that differ per XCD (the default, equal ones and two lopsided sets) change only where the
    contexts are cut; long enough contexts that the weighted split is in effect, ragged ends included."""
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.YI_6B
    kv_lens = [9000, 12001, 7000, 15000, 11007, 13001, 33, 1]
    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed=77)
    scale = W.softmax_scale(shape.head_dim)
    s = _session(shape, n, max(kv_lens))
    reqids = s.load_contexts(inp.k, inp.v)
    if weights is not None:
        assert s.va.set_decode_xcd_weights(weights) == 0, P.last_error()
    got = tensor_to_f32(s.decode(0, bits_to_tensor(inp.q), reqids, kv_lens, scale))
    assert s.va.set_decode_xcd_weights([1, 1, 1, 1, 1, 1, 1, 0.1]) == -1 and "weights" in P.last_error()
    assert s.va.set_decode_xcd_weights(None) == 0
    s.close()
    check(got, OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale), f"decode with XCD weights {weights}")


@pytest.mark.parametrize("per_slot", [2, 5, 64])
def test_decode_invariant_to_segments_per_slot(per_slot):
    """More, shorter segments than resident workgroups (set_decode_tuning): same result, and the workspace the
    library asks for covers them."""
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.LLAMA3_8B
    kv_lens = [9000, 12001, 33, 1, 20000]
    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed=per_slot)
    scale = W.softmax_scale(shape.head_dim)
    s = _session(shape, n, max(kv_lens))
    reqids = s.load_contexts(inp.k, inp.v)
    small = s.va.decode_workspace_bytes(kv_lens)
    assert s.va.set_decode_tuning(per_slot) == 0, P.last_error()
    assert s.va.decode_workspace_bytes(kv_lens) > small
    got = tensor_to_f32(s.decode(0, bits_to_tensor(inp.q), reqids, kv_lens, scale))
    assert s.va.set_decode_tuning(0) == -1 and s.va.set_decode_tuning(65) == -1
    s.close()
    check(got, OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale), f"decode with {per_slot} segments per slot")


@pytest.mark.parametrize("G", [4 * KiB, 64 * KiB, 2 * MiB])
def test_decode_invariant_to_page_group_size(G):
    shape = W.LLAMA3_8B
    kv_lens = [1500, 37, 2600]
    got, want, _ = _run_decode(shape, kv_lens, seed=6, G=G)
    check(got, want, f"decode G={G}")


def test_context_of_one_returns_v_bit_exactly():
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_bits

    shape = W.YI_34B
    inp = W.draw_attention_inputs(shape, [1, 1], [1, 1], seed=9)
    s = _session(shape, 2, 16)
    reqids = s.load_contexts(inp.k, inp.v)
    o = tensor_to_bits(s.decode(0, bits_to_tensor(inp.q), reqids, [1, 1], 0.0884))
    p = tensor_to_bits(s.prefill(0, bits_to_tensor(inp.q), reqids, [0, 1, 2], [1, 1], 0.0884))
    s.close()
    for r in range(2):
        for h in range(shape.num_q_heads):
            assert np.array_equal(o[r, h], inp.v[r][0, h // shape.group])
            assert np.array_equal(p[r, h], inp.v[r][0, h // shape.group])


def _run_prefill(shape, q_lens, kv_lens, seed, G=2 * MiB):
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed)
    scale = W.softmax_scale(shape.head_dim)
    s = _session(shape, len(q_lens), max(kv_lens), G)
    reqids = s.load_contexts(inp.k, inp.v)
    got = tensor_to_f32(s.prefill(0, bits_to_tensor(inp.q), reqids, inp.cu_q, kv_lens, scale))
    s.close()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    return got, want


@pytest.mark.parametrize("Hq,H,D", [(8, 2, 64), (32, 8, 128), (14, 2, 128), (4, 4, 64), (3, 3, 128)])
def test_prefill_shapes_ragged_lengths(Hq, H, D):
    shape = W.Shape("t", Hq, H, D, 1)
    q_lens = [1, 5, 64, 127, 128, 129, 300, 0, 513, 1100]
    got, want = _run_prefill(shape, q_lens, list(q_lens[:7]) + [10, 513, 1100], seed=Hq + D)
    check(got, want, f"prefill Hq={Hq} H={H} D={D}")


def test_prefill_chunk_appended_to_existing_context():
    """A 300-token chunk appended at context 1000 attends to all 1300 tokens (config 4's shape of
    request, scaled down), together with fresh prompts and a decode-like q_len=1 row."""
    shape = W.YI_34B
    got, want = _run_prefill(shape, [300, 200, 1, 77], [1300, 200, 555, 400], seed=12)
    check(got, want, "chunked prefill")


@pytest.mark.parametrize("kind", ["sharp", "flat", "rising", "falling"])
def test_score_ranges_that_stress_the_running_maximum(kind):
    """Value distributions away from N(0,1): scores 16x larger (softmax close to one-hot), 64x smaller (close to a
    mean), and scores that rise or fall steadily along the context, so that the running maximum is raised in every
    tile (or only in the first) and split-K partials carry maxima hundreds of binary orders apart.  Prefill (chunk
    appended to a context) and decode, against the oracle."""
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", 16, 4, 128, 1)
    q_lens, kv_lens = [300, 1, 129], [2300, 4000, 129]
    inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed=31)
    f32 = W.bf16_bits_to_f32
    if kind == "sharp":
        inp.q = W.f32_to_bf16_bits(f32(inp.q) * 16.0)
    elif kind == "flat":
        inp.q = W.f32_to_bf16_bits(f32(inp.q) / 64.0)
    else:
        # q = +-1 in every channel of one sign pattern; keys carry that pattern times a ramp over the positions,
        # so that the score of key t is about 0.7 * (t - L/2) (rising) or its negative: 45 per 64-token tile
        sign = np.where(np.arange(128) % 2 == 0, 1.0, -1.0).astype(np.float32)
        inp.q = W.f32_to_bf16_bits(np.broadcast_to(sign, inp.q.shape).astype(np.float32) * 1.0)
        for r, L in enumerate(kv_lens):
            ramp = ((np.arange(L, dtype=np.float32) - L / 2) * (0.0625 if kind == "rising" else -0.0625))[:, None, None]
            inp.k[r] = W.f32_to_bf16_bits(f32(inp.k[r]) * 0.05 + ramp * sign)
    scale = W.softmax_scale(128)
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    # A near one-hot softmax returns single V rows, with entries up to ~4: the bf16 output's spacing there (2^-6 .. 2^-5)
    # already exceeds the absolute bound meant for outputs of order 0.1.  Rows are therefore compared in units of
    # max(1, largest entry of the row): the absolute bound scales with the row, the relative one is unchanged.
    unit = np.maximum(1.0, np.abs(want).max(axis=-1, keepdims=True))
    s = _session(shape, 3, max(kv_lens))
    ids = s.load_contexts(inp.k, inp.v)
    got = tensor_to_f32(s.prefill(0, bits_to_tensor(inp.q), ids, inp.cu_q, kv_lens, scale))
    check(got / unit, want / unit, f"prefill, {kind} scores")
    # decode: the last query row of every request over its whole context
    last = np.array([int(c) - 1 for c in inp.cu_q[1:]])
    gd = tensor_to_f32(s.decode(0, bits_to_tensor(inp.q[last]), ids, kv_lens, scale))
    check(gd / unit[last], want[last] / unit[last], f"decode, {kind} scores")
    assert s.va.set_decode_chunk(64) == 0          # many partials per request, each with a maximum of its own
    gd = tensor_to_f32(s.decode(0, bits_to_tensor(inp.q[last]), ids, kv_lens, scale))
    check(gd / unit[last], want[last] / unit[last], f"decode in 64-token pieces, {kind} scores")
    s.close()


def test_decode_equals_last_prefill_row_on_gpu():
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.LLAMA3_8B
    L = 700
    inp = W.draw_attention_inputs(shape, [L], [L], seed=13)
    scale = W.softmax_scale(128)
    s = _session(shape, 1, L)
    reqids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    pre = tensor_to_f32(s.prefill(0, q, reqids, [0, L], [L], scale))
    dec = tensor_to_f32(s.decode(0, q[L - 1:L].contiguous(), reqids, [L], scale))
    s.close()
    want = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale, rows=np.array([L - 1], dtype=np.int32))
    check(dec[0], want[0], "decode row")
    check(pre[L - 1], want[0], "prefill last row")


def test_calls_on_another_stream_do_not_disturb_a_running_prefill():
    """A long prefill on stream A is followed at once by more calls on stream B than the library has staging slots for
    index arrays, work queues and queue counters (eight): a slot must stay taken until the kernel that reads it has
    ended - not merely until its upload has - whichever stream asks for it next.  The long prefill's output and the
    short ones' are checked against the oracle, and the scale argument rejects non-positive values on the way."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.LLAMA3_8B
    scale = W.softmax_scale(128)
    big = [9000, 7001]                       # ~1 ms of prefill kernel
    small = [70, 33]
    inp = W.draw_attention_inputs(shape, big + small, big + small, seed=21)
    s = _session(shape, 4, max(big))
    ids = s.load_contexts(inp.k, inp.v)
    torch.cuda.synchronize()
    q = bits_to_tensor(inp.q)
    cu = [int(x) for x in inp.cu_q]
    q_big, q_small = q[:cu[2]].contiguous(), q[cu[2]:].contiguous()
    o_big = torch.empty_like(q_big)
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    assert s.va.attn_prefill(0, a.cuda_stream, q_big, o_big, ids[:2], [0, big[0], big[0] + big[1]], big, scale) == 0, P.last_error()
    for bad in (0.0, -scale, float("nan"), float("inf")):
        assert s.va.attn_prefill(0, b.cuda_stream, q_small, o_big, ids[2:], [0, 70, 103], small, bad) == -1 and "scale" in P.last_error()
    for i in range(12):                      # more than the eight staging slots, all while stream A is still busy
        o = torch.empty_like(q_small)
        assert s.va.attn_prefill(0, b.cuda_stream, q_small, o, ids[2:], [0, 70, 103], small, scale) == 0, P.last_error()
        outs.append(o)
    torch.cuda.synchronize()
    rows = W.sample_rows(big[0], 24, seed=1, boundaries=[384, 385, 8999 - 384])
    want = OA.attention_request(inp.q[:big[0]], inp.k[0], inp.v[0], scale, rows=rows)
    check(tensor_to_f32(o_big[:big[0]])[rows], want, "long prefill on stream A, request 0")
    rows1 = W.sample_rows(big[1], 24, seed=2, boundaries=[256, 7000 - 384])
    want1 = OA.attention_request(inp.q[big[0]:cu[2]], inp.k[1], inp.v[1], scale, rows=rows1)
    check(tensor_to_f32(o_big[big[0]:])[rows1], want1, "long prefill on stream A, request 1")
    want_small = OA.attention_batch(inp.q[cu[2]:], np.array([0, 70, 103]), inp.k[2:], inp.v[2:], scale)
    for i, o in enumerate(outs):
        check(tensor_to_f32(o), want_small, f"short prefill {i} on stream B")
    s.close()


def test_batch_slots_map_to_arbitrary_reqids_with_holes():
    """Continuous batching: after a request in the middle leaves, the remaining batch slots keep
    their reqIds (holes in the virtual tensors) and a newcomer reuses the freed id."""
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.YI_6B
    kv = [400, 90, 1000, 257]
    inp = W.draw_attention_inputs(shape, [1] * 4, kv, seed=14)
    scale = W.softmax_scale(128)
    s = _session(shape, 4, 1024)
    ids = s.load_contexts(inp.k, inp.v)
    s.finish(ids[1])
    new = W.draw_attention_inputs(shape, [1], [333], seed=15)
    nid = s.load_contexts(new.k, new.v)[0]
    assert nid == ids[1]
    order = [3, 0, 1, 2]  # batch slot -> which request; slot 2 is the newcomer
    reqids = [ids[3], ids[0], nid, ids[2]]
    q_bits = np.stack([inp.q[3], inp.q[0], new.q[0], inp.q[2]])
    lens = [kv[3], kv[0], 333, kv[2]]
    got = tensor_to_f32(s.decode(0, bits_to_tensor(q_bits), reqids, lens, scale))
    s.close()
    ks = [inp.k[3], inp.k[0], new.k[0], inp.k[2]]
    vs = [inp.v[3], inp.v[0], new.v[0], inp.v[2]]
    want = OA.attention_batch(q_bits, np.arange(5), ks, vs, scale)
    check(got, want, "holes")


def test_attention_rejects_unbacked_or_inactive_requests():
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor

    shape = W.TINY
    s = _session(shape, 2, 4096, G=64 * KiB)
    inp = W.draw_attention_inputs(shape, [1], [100], seed=16)
    ids = s.load_contexts(inp.k, inp.v)
    q = bits_to_tensor(inp.q)
    o = torch.empty_like(q)
    ws = s.workspace([4096])
    tokens_backed = 64 * KiB // shape.token_bytes
    assert s.va.attn_decode(0, s.stream, q, o, ids, [tokens_backed + 1], 0.1, ws, ws.numel()) == -1
    assert "mapped" in P.last_error()
    assert s.va.attn_decode(0, s.stream, q, o, [1], [10], 0.1, ws, ws.numel()) == -1      # inactive id
    assert s.va.attn_decode(0, s.stream, q, o, ids, [0], 0.1, ws, ws.numel()) == -1       # empty context
    assert s.va.attn_decode(0, s.stream, q, o, ids, [100], 0.1, ws, 16) == -1             # workspace
    assert s.va.attn_prefill(0, s.stream, q, o, ids, [0, 1], [0], 0.1) == -1              # kv_len < q_len
    assert s.va.attn_prefill(1, s.stream, q, o, ids, [0, 1], [100], 0.1) == -1            # layer
    assert s.va.attn_decode(0, s.stream, q, o, ids, [100], 0.1, ws, ws.numel()) == 0
    s.close()


def test_config2_yi6b_decode_full_size_matches_oracle():
    """BASELINE config 2 at full size, in the launch configuration bench.py times (default chunking,
    2 MiB page-groups): every output row checked against the oracle."""
    wl = W.config(1)
    got, want, _ = _run_decode(wl.shape, wl.kv_lens, wl.seed)
    check(got, want, "C2 decode")


@pytest.mark.parametrize("Hq,H,D", [(32, 4, 128), (40, 2, 64), (56, 8, 128)])
def test_decode_with_fused_append_matches_oracle_and_fills_the_cache(Hq, H, D):
    """vattn_attn_decode_append = append_kv + attn_decode in one launch: the newest token's K/V rows are taken
    from the caller's buffers, attended to, and stored at position kv_len-1 of the cache."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", Hq, H, D, 1)
    kv_lens = [1, 2, 32, 33, 64, 65, 1000, 2049, 4096]      # newest token first / last in a tile, alone, across segments
    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed=Hq + D)
    scale = W.softmax_scale(D)
    s = _session(shape, n, max(kv_lens))
    ids = [s.admit(L) for L in kv_lens]
    s.step()
    # the cache holds everything but the newest token of each request; its slot holds a poison pattern
    old_k = [k[:-1] for k in inp.k]
    old_v = [v[:-1] for v in inp.v]
    cu = np.zeros(n + 1, dtype=np.int64); cu[1:] = np.cumsum([L - 1 for L in kv_lens])
    if cu[-1]:
        s.append(0, bits_to_tensor(np.concatenate(old_k)), bits_to_tensor(np.concatenate(old_v)), ids, cu, [0] * n)
    poison = torch.full((n, H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    s.append(0, poison, poison, ids, np.arange(n + 1), [L - 1 for L in kv_lens])
    k_new = bits_to_tensor(np.stack([k[-1] for k in inp.k]))
    v_new = bits_to_tensor(np.stack([v[-1] for v in inp.v]))
    q = bits_to_tensor(inp.q)
    o = torch.empty_like(q)
    ws = s.workspace(kv_lens)
    rc = s.va.attn_decode_append(0, s.stream, q, k_new, v_new, o, ids, kv_lens, scale, ws, ws.numel())
    assert rc == 0, P.last_error()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    check(tensor_to_f32(o), want, "fused append + decode")
    # the cache now holds the new rows: a plain decode over it gives the same answer
    check(tensor_to_f32(s.decode(0, q, ids, kv_lens, scale)), want, "plain decode after the fused append")
    assert s.va.attn_decode_append(0, s.stream, q[:2], k_new[:2], v_new[:2], o[:2], [ids[0], ids[0]], kv_lens[:2], scale, ws, ws.numel()) == -1
    s.close()


@pytest.mark.parametrize("Hq,H,D", [(8, 2, 64), (32, 8, 128), (14, 2, 128)])
def test_prefill_with_fused_append_matches_oracle_and_fills_the_cache(Hq, H, D):
    """vattn_attn_prefill_append = append_kv + attn_prefill in one launch: the K/V rows of the query tokens are
    taken from the caller's buffers, attended to, and stored at positions kv_len-q_len .. kv_len-1.  Chunks that
    start on a tile boundary, inside a tile, at position 0, a single-token chunk and an empty one."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", Hq, H, D, 1)
    q_lens = [300, 200, 1, 77, 0, 513, 129, 64]
    offs = [1000, 0, 554, 323, 10, 64, 63, 1]
    kv_lens = [q + o for q, o in zip(q_lens, offs)]
    n = len(q_lens)
    inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed=Hq + D + 1)
    scale = W.softmax_scale(D)
    s = _session(shape, n, max(kv_lens))
    ids = [s.admit(L) for L in kv_lens]
    s.step()
    # the cache holds the first `off` tokens of each request; the positions of the chunk hold a poison pattern
    cu_old = np.zeros(n + 1, dtype=np.int64); cu_old[1:] = np.cumsum(offs)
    s.append(0, bits_to_tensor(np.concatenate([k[:o] for k, o in zip(inp.k, offs)])),
             bits_to_tensor(np.concatenate([v[:o] for v, o in zip(inp.v, offs)])), ids, cu_old, [0] * n)
    poison = torch.full((int(inp.cu_q[-1]), H, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    s.append(0, poison, poison, ids, inp.cu_q, offs)
    k_new = bits_to_tensor(np.concatenate([k[o:] for k, o in zip(inp.k, offs)]))
    v_new = bits_to_tensor(np.concatenate([v[o:] for v, o in zip(inp.v, offs)]))
    q = bits_to_tensor(inp.q)
    o = torch.empty_like(q)
    rc = s.va.attn_prefill_append(0, s.stream, q, k_new, v_new, o, ids, inp.cu_q, kv_lens, scale)
    assert rc == 0, P.last_error()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    check(tensor_to_f32(o), want, "fused append + prefill")
    # the cache now holds the new rows: a plain prefill over it does the same arithmetic on the same bytes
    o2 = s.prefill(0, q, ids, inp.cu_q, kv_lens, scale)
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16))
    # a reqId with a non-empty chunk may appear only once
    assert s.va.attn_prefill_append(0, s.stream, q[:500], k_new[:500], v_new[:500], o[:500], [ids[0], ids[0]], [0, 300, 500],
                                    [kv_lens[0], kv_lens[0]], scale) == -1
    s.close()


def test_prefill_with_fused_append_in_the_sliced_layout():
    """All layers in one buffer: the cache's tokens are N*H*D apart, the caller's new rows H*D; chunks that start on
    and inside a tile, both layers."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession, bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", 8, 2, 64, 3)
    layers = 3
    q_lens = [300, 129, 1, 64]
    offs = [1000, 0, 77, 64]
    kv_lens = [q + o for q, o in zip(q_lens, offs)]
    n = len(q_lens)
    scale = W.softmax_scale(64)
    G = 64 * KiB
    per_req = (max(kv_lens) * shape.token_bytes * layers + G - 1) // G * G
    s = KvSession(8, 2, 64, n, max(kv_lens), per_req * 2 * n, layers, G, flags=P.FLAG_TENSOR_SLICING)
    ids = [s.admit(L) for L in kv_lens]
    s.step()
    for layer in (2, 0):
        inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed=40 + layer)
        cu_old = np.zeros(n + 1, dtype=np.int64); cu_old[1:] = np.cumsum(offs)
        s.append(layer, bits_to_tensor(np.concatenate([k[:o] for k, o in zip(inp.k, offs)])),
                 bits_to_tensor(np.concatenate([v[:o] for v, o in zip(inp.v, offs)])), ids, cu_old, [0] * n)
        poison = torch.full((int(inp.cu_q[-1]), 2, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
        s.append(layer, poison, poison, ids, inp.cu_q, offs)
        k_new = bits_to_tensor(np.concatenate([k[o:] for k, o in zip(inp.k, offs)]))
        v_new = bits_to_tensor(np.concatenate([v[o:] for v, o in zip(inp.v, offs)]))
        q = bits_to_tensor(inp.q)
        o = torch.empty_like(q)
        assert s.va.attn_prefill_append(layer, s.stream, q, k_new, v_new, o, ids, inp.cu_q, kv_lens, scale) == 0, P.last_error()
        want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
        check(tensor_to_f32(o), want, f"fused append + prefill, sliced layout, layer {layer}")
        o2 = s.prefill(layer, q, ids, inp.cu_q, kv_lens, scale)       # the cache holds the rows now
        assert torch.equal(o.view(torch.int16), o2.view(torch.int16))
    s.close()
