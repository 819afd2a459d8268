"""GPU parity of the attention path under the memory-manager variants: all layers in one buffer
(tensor slicing, strided tokens), statically backed buffers (the hipMalloc baseline), the background
thread, and a sub-tensor larger than 4 GiB (64-bit tile addressing).  Same oracle, same tolerance."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from parity import check

pytestmark = pytest.mark.gpu
KiB, MiB = 1024, 1024 * 1024


def _session(shape, n, max_ctx, layers, G, flags, policy=0, **kw):
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession

    sliced = bool(flags & P.FLAG_TENSOR_SLICING)
    tok = shape.token_bytes * (layers if sliced else 1)
    per_req = (max_ctx * tok + G - 1) // G * G
    budget = per_req * 2 * (1 if sliced else layers) * (n + 2)
    return KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + 2, max_ctx, budget, layers, G, policy,
                     flags=flags, **kw)


def _variants():
    import paper_2405_04437_amd as P

    return {"sliced": P.FLAG_TENSOR_SLICING, "static": P.FLAG_STATIC_BACKING, "background": P.FLAG_BACKGROUND,
            "sliced+background": P.FLAG_TENSOR_SLICING | P.FLAG_BACKGROUND, "sliced+static": P.FLAG_TENSOR_SLICING | P.FLAG_STATIC_BACKING}


@pytest.mark.parametrize("variant", ["sliced", "static", "background", "sliced+background", "sliced+static"])
@pytest.mark.parametrize("Hq,H,D", [(32, 4, 128), (14, 2, 64)])
def test_decode_and_prefill_in_every_layer(variant, Hq, H, D):
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_f32

    flags = _variants()[variant]
    shape = W.Shape("t", Hq, H, D, 3)
    layers = 3
    kv_lens = [1, 33, 700, 2049, 1300]
    q_lens = [1, 33, 64, 300, 1300]      # chunks appended to existing contexts, and whole prompts
    scale = W.softmax_scale(D)
    s = _session(shape, len(kv_lens), max(kv_lens) + 4, layers, 64 * KiB, flags, lookahead_tokens=1)
    ids = [s.admit(L) for L in kv_lens]
    s.step()
    per_layer = []
    for layer in range(layers):   # different data in every layer: a wrong layer offset or stride shows up
        inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed=1000 + layer)
        cu = np.zeros(len(kv_lens) + 1, dtype=np.int64); cu[1:] = np.cumsum(kv_lens)
        s.append(layer, bits_to_tensor(np.concatenate(inp.k)), bits_to_tensor(np.concatenate(inp.v)), ids, cu, [0] * len(ids))
        per_layer.append(inp)
    for layer in range(layers):
        inp = per_layer[layer]
        want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
        got = tensor_to_f32(s.prefill(layer, bits_to_tensor(inp.q), ids, inp.cu_q, kv_lens, scale))
        check(got, want, f"{variant} prefill layer {layer}")
        # decode: the last query row of each request against the same context
        last = np.array([inp.cu_q[i + 1] - 1 for i in range(len(ids))])
        got_d = tensor_to_f32(s.decode(layer, bits_to_tensor(inp.q[last]), ids, kv_lens, scale))
        check(got_d, want[last], f"{variant} decode layer {layer}")
    s.close()


def test_background_growth_is_usable_without_waiting():
    """Decode loop with look-ahead: after the first step every later step finds its page-groups mapped by
    the previous background pass, and the kernels launched meanwhile see correct data."""
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import bits_to_tensor, tensor_to_bits, tensor_to_f32
    import torch

    shape = W.Shape("t", 8, 2, 64, 2)
    G = 4 * KiB                                  # 16 tokens per page-group: growth every 16 steps
    s = _session(shape, 3, 400, 2, G, P.FLAG_BACKGROUND, policy=P.POLICY_DEFERRED, lookahead_tokens=1,
                 eager_page_groups=2, reclaim_threshold_page_groups=4)
    kv_lens = [5, 16, 47]
    inp = W.draw_attention_inputs(shape, [1] * 3, kv_lens, seed=9)
    ids = s.load_contexts(inp.k, inp.v)
    scale = W.softmax_scale(64)
    ks, vs = [k.copy() for k in inp.k], [v.copy() for v in inp.v]
    gen = torch.Generator(device="cuda"); gen.manual_seed(3)
    sync0 = s.va.step_counters()[0]
    for it in range(70):
        nk = torch.randn((3, 2, 64), generator=gen, device="cuda").to(torch.bfloat16)
        nv = torch.randn((3, 2, 64), generator=gen, device="cuda").to(torch.bfloat16)
        q = torch.randn((3, 8, 64), generator=gen, device="cuda").to(torch.bfloat16)
        for r, L in zip(ids, kv_lens):
            s.seq_lens[r] = L + 1
        s.step()
        s.append(0, nk, nv, ids, [0, 1, 2, 3], kv_lens)
        kv_lens = [L + 1 for L in kv_lens]
        o = s.decode(0, q, ids, kv_lens, scale)
        nkb, nvb = tensor_to_bits(nk), tensor_to_bits(nv)
        ks = [np.concatenate([k, nkb[i:i + 1]]) for i, k in enumerate(ks)]
        vs = [np.concatenate([v, nvb[i:i + 1]]) for i, v in enumerate(vs)]
        if it % 9 == 0 or it == 69:
            want = OA.attention_batch(tensor_to_bits(q), np.arange(4), ks, vs, scale)
            check(tensor_to_f32(o), want, f"background decode iteration {it}")
    sync1, bg, *_ = s.va.step_counters()
    assert sync1 == sync0 and bg > 0          # no mapping on the caller's thread after the first step
    s.close()


def test_sub_tensor_beyond_4gib_is_addressed_correctly():
    """All layers in one buffer with Llama-3-8B's shape: a token is 64 KiB of the buffer, a 70 000-token
    context spans 4.3 GiB, so token offsets do not fit 32 bits.  Only sampled rows go to the oracle."""
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import tensor_to_bits, tensor_to_f32
    import torch

    shape = W.LLAMA3_8B
    layers, L, layer = 32, 70000, 29
    s = _session(shape, 1, L + 8, layers, 2 * MiB, P.FLAG_TENSOR_SLICING)
    assert s.va.stats()[1] > 4 * 1024 * MiB
    rid = s.admit(L)
    s.step()
    gen = torch.Generator(device="cuda"); gen.manual_seed(11)
    kb, vb, done = [], [], 0
    while done < L:
        n = min(10000, L - done)
        k = torch.randn((n, 8, 128), generator=gen, device="cuda").to(torch.bfloat16)
        v = torch.randn((n, 8, 128), generator=gen, device="cuda").to(torch.bfloat16)
        s.append(layer, k, v, [rid], [0, n], [done])
        kb.append(tensor_to_bits(k)); vb.append(tensor_to_bits(v))
        done += n
    kb, vb = np.concatenate(kb), np.concatenate(vb)
    scale = W.softmax_scale(128)
    # a 4096-row chunk that ends at the context's end: rows see 65 905 .. 70 000 keys
    ql = 4096
    q = torch.randn((ql, 32, 128), generator=gen, device="cuda").to(torch.bfloat16)
    rows = W.sample_rows(ql, 6, seed=3, boundaries=[128, ql - 129])
    want = OA.attention_request(tensor_to_bits(q), kb, vb, scale, rows=rows)
    o = s.prefill(layer, q, [rid], [0, ql], [L], scale)
    check(tensor_to_f32(o)[rows], want, "prefill beyond 4 GiB")
    od = s.decode(layer, q[ql - 1:ql], [rid], [L], scale)
    check(tensor_to_f32(od), want[-1:], "decode beyond 4 GiB")   # sample_rows always includes the last row
    s.close()


@pytest.mark.parametrize("block_tokens", [32, 64, 256])
@pytest.mark.parametrize("Hq,H,D", [(32, 4, 128), (14, 2, 64)])
def test_paged_comparison_kernel_matches_oracle(block_tokens, Hq, H, D):
    """The paged variant of the decode kernel (block table inside the kernel, for measuring what the paper's
    design avoids) computes the same attention: K/V scattered over a shuffled block pool."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession, bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", Hq, H, D, 1)
    kv_lens = [1, 31, 32, 33, 700, 2049, 1300]
    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, [1] * n, kv_lens, seed=block_tokens + D)
    scale = W.softmax_scale(D)
    blocks_per = [(L + block_tokens - 1) // block_tokens for L in kv_lens]
    max_blocks = max(blocks_per)
    num_blocks = sum(blocks_per) + 5
    rng = np.random.default_rng(7)
    ids = rng.permutation(num_blocks)
    table = np.full((n, max_blocks), -1, dtype=np.int32)   # unused entries stay invalid on purpose
    kpool = np.zeros((num_blocks, block_tokens, H, D), dtype=np.uint16)
    vpool = np.zeros_like(kpool)
    nxt = 0
    for r, L in enumerate(kv_lens):
        for j in range(blocks_per[r]):
            b = int(ids[nxt]); nxt += 1
            table[r, j] = b
            a, e = j * block_tokens, min(L, (j + 1) * block_tokens)
            kpool[b, :e - a] = inp.k[r][a:e]
            vpool[b, :e - a] = inp.v[r][a:e]
    s = KvSession(Hq, H, D, 2, 64, 0, 1, 2 * MiB)          # geometry only: no KV memory of its own is used
    q = bits_to_tensor(inp.q)
    o = torch.empty_like(q)
    kp, vp = bits_to_tensor(kpool), bits_to_tensor(vpool)
    ws = s.workspace(kv_lens)
    rc = s.va.attn_decode_paged(s.stream, q, o, kp, vp, num_blocks, block_tokens, table, kv_lens, scale, ws, ws.numel())
    assert rc == 0, P.last_error()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    check(tensor_to_f32(o), want, f"paged decode block={block_tokens}")
    # rejected on the host: a used table entry outside the pool, a context longer than its table row, a bad block size
    bad = table.copy(); bad[4, 1] = num_blocks
    assert s.va.attn_decode_paged(s.stream, q, o, kp, vp, num_blocks, block_tokens, bad, kv_lens, scale, ws, ws.numel()) == -1
    long = list(kv_lens); long[0] = max_blocks * block_tokens + 1
    assert s.va.attn_decode_paged(s.stream, q, o, kp, vp, num_blocks, block_tokens, table, long, scale, ws, ws.numel()) == -1
    assert s.va.attn_decode_paged(s.stream, q, o, kp, vp, num_blocks, 48, table, kv_lens, scale, ws, ws.numel()) == -1
    s.close()


@pytest.mark.parametrize("block_tokens", [64, 256])
@pytest.mark.parametrize("Hq,H,D", [(32, 8, 128), (14, 2, 64)])
def test_paged_prefill_comparison_kernel_matches_oracle(block_tokens, Hq, H, D):
    """The prefill kernel with a block-table lookup per tile (comparison variant) over a shuffled block pool:
    whole prompts and a chunk appended to an existing context."""
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession, bits_to_tensor, tensor_to_f32

    shape = W.Shape("t", Hq, H, D, 1)
    q_lens = [1, 65, 700, 300]
    kv_lens = [1, 65, 700, 1500]
    n = len(kv_lens)
    inp = W.draw_attention_inputs(shape, q_lens, kv_lens, seed=block_tokens + Hq)
    scale = W.softmax_scale(D)
    blocks_per = [(L + block_tokens - 1) // block_tokens for L in kv_lens]
    max_blocks, num_blocks = max(blocks_per), sum(blocks_per) + 3
    ids = np.random.default_rng(11).permutation(num_blocks)
    table = np.full((n, max_blocks), -1, dtype=np.int32)
    kpool = np.zeros((num_blocks, block_tokens, H, D), dtype=np.uint16)
    vpool = np.zeros_like(kpool)
    nxt = 0
    for r, L in enumerate(kv_lens):
        for j in range(blocks_per[r]):
            b = int(ids[nxt]); nxt += 1
            table[r, j] = b
            a, e = j * block_tokens, min(L, (j + 1) * block_tokens)
            kpool[b, :e - a] = inp.k[r][a:e]
            vpool[b, :e - a] = inp.v[r][a:e]
    s = KvSession(Hq, H, D, 2, 64, 0, 1, 2 * MiB)
    q = bits_to_tensor(inp.q)
    o = torch.empty_like(q)
    kp, vp = bits_to_tensor(kpool), bits_to_tensor(vpool)
    rc = s.va.attn_prefill_paged(s.stream, q, o, kp, vp, num_blocks, block_tokens, table, inp.cu_q, kv_lens, scale)
    assert rc == 0, P.last_error()
    want = OA.attention_batch(inp.q, inp.cu_q, inp.k, inp.v, scale)
    check(tensor_to_f32(o), want, f"paged prefill block={block_tokens}")
    bad = table.copy(); bad[2, 0] = -1
    assert s.va.attn_prefill_paged(s.stream, q, o, kp, vp, num_blocks, block_tokens, bad, inp.cu_q, kv_lens, scale) == -1
    assert s.va.attn_prefill_paged(s.stream, q, o, kp, vp, num_blocks, 32, table, inp.cu_q, kv_lens, scale) == -1
    s.close()
