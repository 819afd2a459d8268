"""Algorithm 1 of the paper end to end on the GPU: requests arrive, are prefilled (KV append fused into the prefill
kernel), decode one token per iteration (append fused into the decode kernel), finish and hand their reqId - and,
under the deferred policy, their still-mapped pages with the previous occupant's K/V in them - to the next
arrival.  Every iteration's attention output is checked against the CPU oracle, which is fed from host-side copies
of each request's own K/V only, so anything leaking from a previous occupant or from beyond a context shows up."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from parity import check

pytestmark = pytest.mark.gpu
KiB = 1024


@pytest.mark.parametrize("policy,flags,lookahead", [("sync", 0, 0), ("deferred", 0, 0), ("deferred", "background", 48),
                                                    ("deferred", "background+sliced", 16)])
def test_serving_loop_with_arrivals_and_departures(policy, flags, lookahead):
    import torch
    import paper_2405_04437_amd as P
    from paper_2405_04437_amd.runtime import KvSession, bits_to_tensor, tensor_to_f32

    shape = W.Shape("loop", 8, 2, 64, 2)
    H, D, Hq, layers, B = 2, 64, 8, 2, 6
    G = 16 * KiB                                   # 64 tokens per page-group: plenty of boundary crossings
    max_ctx = 700
    sliced = isinstance(flags, str) and "sliced" in flags
    fl = 0
    if isinstance(flags, str):
        fl |= P.FLAG_BACKGROUND
        if sliced:
            fl |= P.FLAG_TENSOR_SLICING
    per_req = (max_ctx * shape.token_bytes * (layers if sliced else 1) + G - 1) // G * G
    pool = per_req * (2 if sliced else 2 * layers) * B
    s = KvSession(Hq, H, D, B, max_ctx, pool, layers, G, P.POLICY_DEFERRED if policy == "deferred" else P.POLICY_SYNC_UNMAP,
                  flags=fl, lookahead_tokens=lookahead, eager_page_groups=2 if fl else 0,
                  reclaim_threshold_page_groups=4 if fl else 0)
    scale = W.softmax_scale(D)
    rng = np.random.default_rng(11)
    events = W.serving_trace(seed=5, max_batch=B, iterations=40, prompt_range=(1, 300), out_range=(1, 25), arrival_p=0.6)
    live = {}            # reqId -> dict(k=[layers][len,H,D] bits, v=..., left=tokens still to generate)
    waiting = []

    def rows(n):
        return W.normal_bf16(rng, (n, H, D))

    checked = 0
    for kind, prompt, out_len in events:
        if kind == "arrive":
            waiting.append((prompt, out_len))
            continue
        # ---- one iteration: admit what fits, step(), prefill the newcomers, decode the others, retire the finished
        fresh = []
        while waiting and len(live) < B:
            prompt, out_len = waiting.pop(0)
            r = s.va.alloc_reqid()
            assert r >= 0
            live[r] = {"k": [rows(prompt) for _ in range(layers)], "v": [rows(prompt) for _ in range(layers)], "left": out_len, "new": True}
            fresh.append(r)
        running = [r for r in live if r not in fresh]
        for r in running:                          # each running request gets one more token in every layer
            for layer in range(layers):
                live[r]["k"][layer] = np.concatenate([live[r]["k"][layer], rows(1)])
                live[r]["v"][layer] = np.concatenate([live[r]["v"][layer], rows(1)])
        seq = [0] * B
        for r, st in live.items():
            seq[r] = st["k"][0].shape[0]
        assert s.va.step(seq) == 0, P.last_error()
        for layer in range(layers):
            if fresh:
                q_lens = [live[r]["k"][layer].shape[0] for r in fresh]
                cu = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
                q = W.normal_bf16(rng, (int(cu[-1]), Hq, D))
                qt = bits_to_tensor(q)
                o = torch.empty_like(qt)
                kn = bits_to_tensor(np.concatenate([live[r]["k"][layer] for r in fresh]))
                vn = bits_to_tensor(np.concatenate([live[r]["v"][layer] for r in fresh]))
                assert s.va.attn_prefill_append(layer, s.stream, qt, kn, vn, o, fresh, cu, q_lens, scale) == 0, P.last_error()
                want = OA.attention_batch(q, cu, [live[r]["k"][layer] for r in fresh], [live[r]["v"][layer] for r in fresh], scale)
                check(tensor_to_f32(o), want, f"prefill of {fresh} in layer {layer}")
                checked += 1
            if running:
                n = len(running)
                kv_lens = [live[r]["k"][layer].shape[0] for r in running]
                q = W.normal_bf16(rng, (n, Hq, D))
                qt = bits_to_tensor(q)
                o = torch.empty_like(qt)
                kn = bits_to_tensor(np.stack([live[r]["k"][layer][-1] for r in running]))
                vn = bits_to_tensor(np.stack([live[r]["v"][layer][-1] for r in running]))
                ws = s.workspace(kv_lens)
                assert s.va.attn_decode_append(layer, s.stream, qt, kn, vn, o, running, kv_lens, scale, ws, ws.numel()) == 0, P.last_error()
                want = OA.attention_batch(q, np.arange(n + 1), [live[r]["k"][layer] for r in running], [live[r]["v"][layer] for r in running], scale)
                check(tensor_to_f32(o), want, f"decode of {running} in layer {layer}")
                checked += 1
        torch.cuda.synchronize()
        for r in list(live):
            live[r]["left"] -= 1
            if live[r]["left"] <= 0 or live[r]["k"][0].shape[0] + 1 >= max_ctx:
                assert s.va.free_reqid(r) == 0
                del live[r]
    assert checked > 60
    s.close()
