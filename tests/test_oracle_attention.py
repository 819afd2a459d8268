"""Pins for the CPU attention oracle: it is checked against things other than itself.

Each test names what fixes the expected value: the definition evaluated by brute force in pure
Python, closed forms of softmax attention, a library SDPA routine as a special case, and the
invariants the definition implies (rows of the softmax sum to 1, a context of one token returns V,
the result does not depend on how the context was chunked).
"""
import math

import numpy as np
import pytest

import workloads as W
from oracle import attention as OA


def _draw(shape, q_lens, kv_lens, seed):
    return W.draw_attention_inputs(shape, q_lens, kv_lens, seed)


def _f(bits):
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def brute_force(q, k, v, scale):
    """Eq. 2 with explicit Python loops and Python floats (no numpy arithmetic)."""
    qf, kf, vf = _f(q).tolist(), _f(k).tolist(), _f(v).tolist()
    q_len, Hq, D = q.shape
    kv_len, H, _ = k.shape
    g = Hq // H
    out = np.zeros((q_len, Hq, D))
    for i in range(q_len):
        n = kv_len - q_len + i + 1
        for h in range(Hq):
            kvh = h // g
            s = []
            for j in range(n):
                acc = 0.0
                for d in range(D):
                    acc += qf[i][h][d] * kf[j][kvh][d]
                s.append(acc * scale)
            m = max(s)
            e = [math.exp(x - m) for x in s]
            z = math.fsum(e)
            for d in range(D):
                out[i, h, d] = math.fsum(e[j] * vf[j][kvh][d] for j in range(n)) / z
    return out


@pytest.mark.parametrize("Hq,H,D", [(1, 1, 64), (4, 1, 64), (7, 1, 128), (8, 2, 128), (14, 2, 64)])
@pytest.mark.parametrize("q_len,kv_len", [(1, 1), (1, 37), (5, 5), (6, 19)])
def test_brute_force_tiny(Hq, H, D, q_len, kv_len):
    shape = W.Shape("t", Hq, H, D, 1)
    inp = _draw(shape, [q_len], [kv_len], seed=Hq * 1000 + D + q_len * 7 + kv_len)
    scale = W.softmax_scale(D)
    got = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale)
    want = brute_force(inp.q, inp.k[0], inp.v[0], scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_softmax_rows_sum_to_one_and_are_positive():
    shape = W.Shape("t", 8, 2, 64, 1)
    inp = _draw(shape, [1], [300], seed=11)
    for kvh in range(2):
        p = OA.softmax_row(inp.q[0, kvh * 4], inp.k[0], kvh, W.softmax_scale(64))
        assert abs(p.sum() - 1.0) < 1e-12
        assert (p > 0).all() and p.shape == (300,)


def test_softmax_matches_independent_formula():
    shape = W.Shape("t", 2, 2, 128, 1)
    inp = _draw(shape, [1], [64], seed=5)
    scale = 0.3
    s = (_f(inp.k[0])[:, 1, :] @ _f(inp.q[0, 1])) * scale
    want = np.exp(s - np.logaddexp.reduce(s))  # exp(s - logsumexp(s))
    got = OA.softmax_row(inp.q[0, 1], inp.k[0], 1, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_context_of_one_returns_v_exactly():
    shape = W.Shape("t", 8, 2, 64, 1)
    inp = _draw(shape, [1], [1], seed=3)
    out = OA.attention_request(inp.q, inp.k[0], inp.v[0], 0.125)
    vf = _f(inp.v[0])
    for h in range(8):
        assert np.array_equal(out[0, h], vf[0, h // 4])


def test_library_sdpa_special_case():
    """PyTorch's CPU scaled_dot_product_attention in float64 with an explicit boolean mask and KV
    heads repeated for the group: a library routine, used here only as a second opinion."""
    import torch

    shape = W.Shape("t", 8, 2, 128, 1)
    q_len, kv_len = 33, 97
    inp = _draw(shape, [q_len], [kv_len], seed=21)
    scale = W.softmax_scale(128)
    got = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale)
    q = torch.from_numpy(_f(inp.q)).permute(1, 0, 2)                      # [Hq, q, D]
    k = torch.from_numpy(_f(inp.k[0])).permute(1, 0, 2).repeat_interleave(4, dim=0)
    v = torch.from_numpy(_f(inp.v[0])).permute(1, 0, 2).repeat_interleave(4, dim=0)
    i = torch.arange(q_len)[:, None]
    j = torch.arange(kv_len)[None, :]
    mask = j <= (kv_len - q_len + i)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(got, ref.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_identical_keys_give_mean_of_values():
    shape = W.Shape("t", 4, 2, 64, 1)
    inp = _draw(shape, [1], [50], seed=8)
    k = np.repeat(inp.k[0][:1], 50, axis=0)
    out = OA.attention_request(inp.q, k, inp.v[0], 0.2)
    vf = _f(inp.v[0])
    for h in range(4):
        np.testing.assert_allclose(out[0, h], vf[:, h // 2].mean(axis=0), rtol=1e-12, atol=1e-14)


def test_constant_values_give_that_constant():
    shape = W.Shape("t", 4, 4, 64, 1)
    inp = _draw(shape, [3], [9], seed=9)
    v = np.full_like(inp.v[0], W.f32_to_bf16_bits(np.array([1.5], dtype=np.float32))[0])
    out = OA.attention_request(inp.q, inp.k[0], v, 0.125)
    np.testing.assert_allclose(out, 1.5, rtol=1e-13)


def test_dominant_key_selects_its_value_row():
    shape = W.Shape("t", 2, 1, 64, 1)
    inp = _draw(shape, [1], [20], seed=10)
    k = inp.k[0].copy()
    k[7, 0] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(inp.q[0, 0]) * 64.0)  # score >> all others
    out = OA.attention_request(inp.q[:, :1], k, inp.v[0], 1.0)
    np.testing.assert_allclose(out[0, 0], _f(inp.v[0])[7, 0], atol=1e-12)


def test_decode_is_invariant_to_token_order():
    shape = W.Shape("t", 8, 2, 64, 1)
    inp = _draw(shape, [1], [123], seed=12)
    perm = np.random.default_rng(0).permutation(123)
    a = OA.attention_request(inp.q, inp.k[0], inp.v[0], 0.125)
    b = OA.attention_request(inp.q, inp.k[0][perm], inp.v[0][perm], 0.125)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_shift_invariance_of_scores():
    """Adding the same vector c to every key changes all scores of a row by q.c: softmax, and so
    the output, is unchanged."""
    shape = W.Shape("t", 1, 1, 64, 1)
    inp = _draw(shape, [1], [40], seed=13)
    kf = W.bf16_bits_to_f32(inp.k[0])
    c = np.zeros(64, dtype=np.float32)
    c[3] = 2.0  # power of two, small: k + c stays exactly representable for most entries
    k2 = W.f32_to_bf16_bits(kf + c)
    # compare against the definition evaluated on the shifted keys rather than assume exactness
    a = OA.attention_request(inp.q, k2, inp.v[0], 0.125)
    b = brute_force(inp.q, k2, inp.v[0], 0.125)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    # and with exactly shifted keys in double precision the softmax itself is unchanged
    s = (kf[:, 0, :].astype(np.float64) @ _f(inp.q[0, 0])) * 0.125
    s2 = ((kf[:, 0, :].astype(np.float64) + c) @ _f(inp.q[0, 0])) * 0.125
    p1 = np.exp(s - s.max()); p1 /= p1.sum()
    p2 = np.exp(s2 - s2.max()); p2 /= p2.sum()
    np.testing.assert_allclose(p1, p2, rtol=1e-9)


def test_heads_of_one_group_with_equal_queries_agree():
    shape = W.Shape("t", 8, 2, 64, 1)
    inp = _draw(shape, [2], [31], seed=14)
    q = inp.q.copy()
    q[:, 1] = q[:, 0]; q[:, 2] = q[:, 0]; q[:, 3] = q[:, 0]
    out = OA.attention_request(q, inp.k[0], inp.v[0], 0.125)
    for h in (1, 2, 3):
        assert np.array_equal(out[:, h], out[:, 0])
    assert not np.array_equal(out[:, 4], out[:, 0])  # other KV head


def test_prefill_is_invariant_to_chunking():
    """One-shot prefill of 48 tokens == prefill of 32 tokens followed by a 16-token chunk that
    attends to all 48 (the bottom-right aligned causal mask)."""
    shape = W.Shape("t", 4, 2, 64, 1)
    inp = _draw(shape, [48], [48], seed=15)
    scale = W.softmax_scale(64)
    whole = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale)
    first = OA.attention_request(inp.q[:32], inp.k[0][:32], inp.v[0][:32], scale)
    second = OA.attention_request(inp.q[32:], inp.k[0], inp.v[0], scale)
    np.testing.assert_allclose(whole[:32], first, rtol=1e-13, atol=0)
    np.testing.assert_allclose(whole[32:], second, rtol=1e-13, atol=0)


def test_decode_equals_last_prefill_row_and_row_subset():
    shape = W.Shape("t", 8, 2, 64, 1)
    inp = _draw(shape, [40], [40], seed=16)
    scale = W.softmax_scale(64)
    whole = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale)
    dec = OA.attention_request(inp.q[39:40], inp.k[0], inp.v[0], scale)
    assert np.array_equal(whole[39], dec[0])
    rows = np.array([0, 17, 39], dtype=np.int32)
    sub = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale, rows=rows)
    assert np.array_equal(sub, whole[rows])


def test_split_context_merge_identity():
    """Decode over a context split in two parts and merged with the log-sum-exp rule gives the
    one-pass result: the property the split-K path relies on, checked on the oracle itself."""
    shape = W.Shape("t", 2, 1, 64, 1)
    inp = _draw(shape, [1], [90], seed=17)
    scale = W.softmax_scale(64)
    full = OA.attention_request(inp.q, inp.k[0], inp.v[0], scale)
    parts = []
    for a, b in ((0, 50), (50, 90)):
        o = OA.attention_request(inp.q, inp.k[0][a:b], inp.v[0][a:b], scale)
        s = (_f(inp.k[0][a:b])[:, 0, :] @ _f(inp.q[0]).T) * scale  # [tokens, heads]
        lse = np.logaddexp.reduce(s, axis=0)
        parts.append((o[0], lse))
    lse_all = np.logaddexp(parts[0][1], parts[1][1])
    merged = sum(o * np.exp(l - lse_all)[:, None] for o, l in parts)
    np.testing.assert_allclose(merged, full[0], rtol=1e-11, atol=1e-13)


def test_rejects_bad_arguments():
    shape = W.Shape("t", 4, 2, 64, 1)
    inp = _draw(shape, [4], [4], seed=18)
    with pytest.raises(ValueError):
        OA.attention_request(inp.q, inp.k[0][:3], inp.v[0][:3], 1.0)  # kv_len < q_len
    with pytest.raises(ValueError):
        OA.attention_request(inp.q, inp.k[0], inp.v[0], 1.0, rows=np.array([4], dtype=np.int32))


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.140625, 65504.0], dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: nearest-even keeps 1.0
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0078125
    assert back[3] == -2.5 and back[4] == 3.140625
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, t)
