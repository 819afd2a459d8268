#!/usr/bin/env python3
"""Measurements around the memory manager on one MI355X, printed as markdown:

  1. per-call latency of the HIP virtual-memory API at several page-group sizes (the analogue of the
     paper's table of VMM API latencies) and the allocation bandwidth that follows from it (the
     analogue of its allocation-bandwidth table);
  2. page-group size effect: the same decode kernel over KV mapped with 64 KiB / 2 MiB page-groups and
     over a statically backed hipMalloc buffer (the paper's "no TLB thrashing with small pages" check);
  3. latency hiding: a decode loop whose requests cross a page-group boundary every few steps, with
     step() mapping synchronously vs the background thread mapping one step ahead (per-iteration step()
     time, its maximum, and where the map calls happened);
  4. deferred reclamation + eager allocation: time from "request arrives" to "prefill may start"
     (alloc_reqid + step) with pages unmapped on free, deferred, and deferred + eager;
  5. the decode kernel over contiguous KV vs its paged comparison variant (block table inside the kernel);
  6. the decode kernel over the all-layers-in-one-buffer layout (tensor slicing, strided tokens);
  7. internal fragmentation per page-group size and layout.

Everything runs through the C ABI (paper_2405_04437_amd.binding); no result is checked here - parity lives in
tests/.  Usage: python vmm_report.py [--quick]
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
KiB, MiB = 1024, 1024 * 1024
CALLS = ["hipMemAddressReserve", "hipMemCreate", "hipMemMap", "hipMemSetAccess (per page-group)",
         "hipMemSetAccess (one call, all)", "hipMemUnmap", "hipMemRelease", "hipMemAddressFree", "touch kernel (all)"]


def api_latency(P, quick):
    sizes = [(4 * KiB, 256), (64 * KiB, 256), (256 * KiB, 256), (2 * MiB, 256), (32 * MiB, 32)]
    rows = {}
    for G, count in sizes:
        if quick:
            count = min(count, 32)
        best = None
        for _ in range(3):
            us = P.vmm_microbench(G, count)
            best = us if best is None else [min(a, b) for a, b in zip(best, us)]
        rows[G] = (count, best)
    print("## 1. HIP virtual-memory API latency (microseconds per call, best of 3 runs)\n")
    print("| call | " + " | ".join(f"{G // KiB} KiB" for G, _ in sizes) + " |")
    print("|---|" + "---|" * len(sizes))
    for i, name in enumerate(CALLS):
        print(f"| {name} | " + " | ".join(f"{rows[G][1][i]:.1f}" for G, _ in sizes) + " |")
    for i, name in ((9, "memory mappings of the process added per hipMemCreate"), (10, "... added per hipMemMap"),
                    (11, "... given back per hipMemUnmap")):
        print(f"| {name} | " + " | ".join(f"{rows[G][1][i]:.2f}" for G, _ in sizes) + " |")
    print("\nPage-groups per run: " + ", ".join(f"{G // KiB} KiB x {rows[G][0]}" for G, _ in sizes))
    print("\nAllocation bandwidth = page-group bytes / (hipMemMap + hipMemSetAccess per page-group):\n")
    print("| page-group | us per page-group | GB/s |")
    print("|---|---|---|")
    for G, _ in sizes:
        t = rows[G][1][2] + rows[G][1][3]
        print(f"| {G // KiB} KiB | {t:.1f} | {G / t / 1e3:.2f} |")
    print()


def _decode_session(P, torch, W, G, flags, n=32, ctx=8192, layers=2):
    from paper_2405_04437_amd.runtime import KvSession

    shape = W.YI_6B
    max_ctx = ctx + 4096
    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    s = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + 4, max_ctx, per_req * 2 * layers * (n + 4), layers, G,
                  P.POLICY_DEFERRED, flags=flags, lookahead_tokens=1)
    gen = torch.Generator(device="cuda"); gen.manual_seed(1)
    ids = [s.admit(ctx) for _ in range(n)]
    s.step()
    for r in ids:
        for layer in range(layers):
            k = torch.randn((ctx, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
            s.append(layer, k, k, [r], [0, ctx], [0])
    return s, ids, shape, gen


def page_size_effect(P, torch, W, quick):
    print("## 2. Page-group size vs decode kernel bandwidth (32 requests x 8192 tokens, Yi-6B shape)\n")
    print("| backing | split-K kernel us | GB/s |")
    print("|---|---|---|")
    for name, G, flags in (("VMM, 64 KiB page-groups", 64 * KiB, 0), ("VMM, 256 KiB page-groups", 256 * KiB, 0),
                           ("VMM, 2 MiB page-groups", 2 * MiB, 0), ("hipMalloc (static backing)", 2 * MiB, P.FLAG_STATIC_BACKING)):
        s, ids, shape, gen = _decode_session(P, torch, W, G, flags)
        n, ctx = len(ids), 8192
        q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        o = torch.empty_like(q)
        lens = [ctx] * n
        ws = s.workspace(lens)
        scale = W.softmax_scale(shape.head_dim)
        for i in range(20):
            s.decode(i % 2, q, ids, lens, scale, out=o, ws=ws)
        torch.cuda.synchronize()
        s.va.set_timing(True); s.va.kernel_time(0)
        for i in range(100):
            s.decode(i % 2, q, ids, lens, scale, out=o, ws=ws)
        torch.cuda.synchronize()
        ms, cnt = s.va.kernel_time(0)
        us = ms * 1e3 / cnt
        nbytes = n * ctx * 2 * shape.token_bytes
        print(f"| {name} | {us:.1f} | {nbytes / us / 1e3:.0f} |")
        s.close()
    print()


def paged_overhead(P, torch, W, quick):
    print("## 5. Paged vs contiguous KV in the same decode kernel (Yi-6B shape, 32 requests x 8192 tokens)\n")
    print("The paged variant looks every 32-token tile up in a block table (blocks scattered over a shuffled pool);")
    print("the contiguous one adds the tile offset to the request's base pointer.\n")
    print("| KV layout | split-K kernel us | GB/s |")
    print("|---|---|---|")
    shape = W.YI_6B
    n, ctx = 32, 8192
    s, ids, shape, gen = _decode_session(P, torch, W, 2 * MiB, 0, n=n, ctx=ctx, layers=1)
    q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    o = torch.empty_like(q)
    lens = [ctx] * n
    ws = s.workspace(lens)
    scale = W.softmax_scale(shape.head_dim)
    nbytes = n * ctx * 2 * shape.token_bytes

    def timed(fn):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        s.va.set_timing(True); s.va.kernel_time(0)
        for _ in range(100):
            fn()
        torch.cuda.synchronize()
        ms, cnt = s.va.kernel_time(0)
        s.va.set_timing(False)
        return ms * 1e3 / cnt

    us = timed(lambda: s.decode(0, q, ids, lens, scale, out=o, ws=ws))
    print(f"| contiguous (virtual tensor) | {us:.1f} | {nbytes / us / 1e3:.0f} |")
    rng = np.random.default_rng(3)
    for bt in (32, 64, 256, 2048):
        per = ctx // bt
        nb = n * per
        pool_k = torch.randn((nb, bt, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        pool_v = torch.randn((nb, bt, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        table = rng.permutation(nb).astype(np.int32).reshape(n, per)
        stream = s.stream
        us = timed(lambda: s.va.attn_decode_paged(stream, q, o, pool_k, pool_v, nb, bt, table, lens, scale, ws, ws.numel()))
        print(f"| paged, {bt}-token blocks | {us:.1f} | {nbytes / us / 1e3:.0f} |")
        del pool_k, pool_v
    s.close()
    print()
    print("Prefill (Llama-3-8B shape, one 16384-token prompt), same kernel with and without the block-table lookup:\n")
    print("| KV layout | prefill kernel ms | TFLOP/s (causal flops) |")
    print("|---|---|---|")
    from paper_2405_04437_amd.runtime import KvSession

    shape = W.LLAMA3_8B
    L = 16384
    flops = 4 * shape.num_q_heads * shape.head_dim * (L * (L + 1) // 2)
    G = 2 * MiB
    per = (L * shape.token_bytes + G - 1) // G * G
    s = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, 1, L, per * 2, 1, G)
    gen = torch.Generator(device="cuda"); gen.manual_seed(2)
    rid = s.admit(L); s.step()
    kv = torch.randn((L, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    s.append(0, kv, kv, [rid], [0, L], [0])
    q = torch.randn((L, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    o = torch.empty_like(q)
    scale = W.softmax_scale(shape.head_dim)

    def timed_p(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        s.va.set_timing(True); s.va.kernel_time(1)
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        ms, cnt = s.va.kernel_time(1)
        s.va.set_timing(False)
        return ms / cnt

    ms = timed_p(lambda: s.prefill(0, q, [rid], [0, L], [L], scale, out=o))
    print(f"| contiguous (virtual tensor) | {ms:.3f} | {flops / ms / 1e9:.0f} |")
    stream = s.stream
    for bt in (64, 256, 2048):
        nb = L // bt
        pool = kv.reshape(nb, bt, shape.num_kv_heads, shape.head_dim)
        perm = rng.permutation(nb)
        shuffled = torch.empty_like(pool)
        shuffled[torch.from_numpy(perm).cuda()] = pool          # logical block j lives in pool slot perm[j]
        table = perm.astype(np.int32).reshape(1, nb)
        ms = timed_p(lambda: s.va.attn_prefill_paged(stream, q, o, shuffled, shuffled, nb, bt, table, [0, L], [L], scale))
        print(f"| paged, {bt}-token blocks | {ms:.3f} | {flops / ms / 1e9:.0f} |")
    ms = timed_p(lambda: s.prefill(0, q, [rid], [0, L], [L], scale, out=o))
    print(f"| contiguous, measured again at the end | {ms:.3f} | {flops / ms / 1e9:.0f} |")
    s.close()
    print()


def slicing_effect(P, torch, W, quick):
    print("## 6. Tensor slicing: decode kernel over [L, N, H, D] (all layers in one buffer) vs [L, H, D] per layer\n")
    print("Yi-6B shape, 32 requests x 4096 tokens, 2 MiB page-groups.  With N layers in one buffer consecutive tokens of")
    print("a layer are N KiB apart and a page-group holds 2048/N tokens of every layer.\n")
    print("| layout | tokens per page-group | page-groups mapped (all buffers) | split-K kernel us | GB/s |")
    print("|---|---|---|---|---|")
    from paper_2405_04437_amd.runtime import KvSession

    shape = W.YI_6B
    n, ctx, G = 32, 4096, 2 * MiB
    for name, layers, flags in (("per-layer buffers, N = 8", 8, 0), ("one buffer, N = 8", 8, P.FLAG_TENSOR_SLICING),
                                ("one buffer, N = 32", 32, P.FLAG_TENSOR_SLICING)):
        sliced = bool(flags)
        tok = shape.token_bytes * (layers if sliced else 1)
        per_req = ((ctx + 64) * tok + G - 1) // G * G
        s = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n, ctx + 64,
                      per_req * 2 * (1 if sliced else layers) * n, layers, G, flags=flags)
        gen = torch.Generator(device="cuda"); gen.manual_seed(1)
        ids = [s.admit(ctx) for _ in range(n)]
        s.step()
        k = torch.randn((ctx, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        for r in ids:
            for layer in (0, layers - 1):
                s.append(layer, k, k, [r], [0, ctx], [0])
        q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        o = torch.empty_like(q)
        lens = [ctx] * n
        ws = s.workspace(lens)
        scale = W.softmax_scale(shape.head_dim)
        for i in range(20):
            s.decode((layers - 1) * (i & 1), q, ids, lens, scale, out=o, ws=ws)
        torch.cuda.synchronize()
        s.va.set_timing(True); s.va.kernel_time(0)
        for i in range(100):
            s.decode((layers - 1) * (i & 1), q, ids, lens, scale, out=o, ws=ws)
        torch.cuda.synchronize()
        ms, cnt = s.va.kernel_time(0)
        us = ms * 1e3 / cnt
        nbytes = n * ctx * 2 * shape.token_bytes
        mapped = s.va.counters()[0]
        print(f"| {name} | {G // tok} | {mapped} | {us:.1f} | {nbytes / us / 1e3:.0f} |")
        s.close()
    print()


def fragmentation(P, W, quick):
    print("## 7. Internal fragmentation: physical memory mapped vs KV bytes in use\n")
    print("32 requests with the context lengths of the Yi-6B decode workload (U[1024,16384]), 2 layers; what step() has")
    print("mapped once every request is backed.  One buffer for all layers (tensor slicing) divides the waste per")
    print("request by the number of layers.\n")
    print("| layout | page-group | tokens per page-group | mapped MiB | in use MiB | wasted | wasted per request KiB |")
    print("|---|---|---|---|---|---|---|")
    from paper_2405_04437_amd.binding import Vattn

    shape = W.YI_6B
    wl = W.config(1)
    lens = [int(x) for x in wl.kv_lens[:32]]
    N, B = 2, 32
    in_use = sum(lens) * shape.token_bytes * 2 * N
    for name, G, flags in (("per-layer buffers", 64 * KiB, 0), ("per-layer buffers", 256 * KiB, 0), ("per-layer buffers", 2 * MiB, 0),
                           ("one buffer for all layers", 2 * MiB, P.FLAG_TENSOR_SLICING)):
        tok = shape.token_bytes * (N if flags else 1)
        per_req = (16384 * tok + G - 1) // G * G
        va = Vattn(N, B, 16384, shape.num_q_heads, shape.num_kv_heads, shape.head_dim, per_req * (2 if flags else 2 * N) * B, G,
                   flags=flags)
        seq = np.zeros(B, dtype=np.int64)
        for L in lens:
            seq[va.alloc_reqid()] = L
        assert va.step(seq) == 0
        Gb, S, total, free = va.stats()
        mapped = (total - free) * Gb
        print(f"| {name} | {G // KiB} KiB | {G // tok} | {mapped / MiB:.1f} | {in_use / MiB:.1f} | {100 * (mapped - in_use) / mapped:.1f} % | {(mapped - in_use) / B / KiB:.0f} |")
        va.destroy()
    print()


def latency_hiding(P, torch, W, quick):
    print("## 3. Synchronous step() vs background look-ahead (decode loop, 32 requests, 256 KiB page-groups)\n")
    print("Every request crosses a page-group boundary every 256 tokens; the 32 requests start at staggered offsets, so")
    print("every 8th step one request needs a new page-group in each of the 2N buffers.  An iteration is step(), the")
    print("KV append and the decode attention of ALL N layers (no other model work: the shortest iteration a serving")
    print("loop could have, i.e. the least time to hide the mapping in), then a stream synchronisation.\n")
    print("| N layers | mode | iteration us | step() mean us | p99 us | max us | map calls in step() | in background | wait for pass us/step |")
    print("|---|---|---|---|---|---|---|---|---|")
    steps = 200 if quick else 1000
    for layers in (2, 8):
        for name, flags in (("synchronous", 0), ("background thread, look-ahead 1", P.FLAG_BACKGROUND)):
            s, ids, shape, gen = _decode_session(P, torch, W, 256 * KiB, flags, ctx=4096, layers=layers)
            n = len(ids)
            lens = np.array([4096 + 8 * i for i in range(n)], dtype=np.int64)
            seq = np.zeros(s.B, dtype=np.int64)
            seq[ids] = lens
            assert s.va.step(seq) == 0
            q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
            knew = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
            o = torch.empty_like(q)
            ws = s.workspace([int(x) + steps + 8 for x in lens])
            scale = W.softmax_scale(shape.head_dim)
            cu = np.arange(n + 1, dtype=np.int32)
            ids_np = np.array(ids, dtype=np.int32)
            c0 = s.va.step_counters()
            times = []
            stream = s.stream
            t_loop = time.perf_counter()
            for i in range(steps):
                seq[ids] = lens + 1
                t0 = time.perf_counter()
                assert s.va.step(seq) == 0
                times.append((time.perf_counter() - t0) * 1e6)
                for layer in range(layers):
                    s.va.append_kv(layer, stream, knew, knew, ids_np, cu, lens)
                lens += 1
                for layer in range(layers):
                    s.va.attn_decode(layer, stream, q, o, ids_np, lens, scale, ws, ws.numel())
                torch.cuda.current_stream().synchronize()
            it_us = (time.perf_counter() - t_loop) * 1e6 / steps
            c1 = s.va.step_counters()
            t = np.array(times)
            print(f"| {layers} | {name} | {it_us:.0f} | {t.mean():.1f} | {np.percentile(t, 99):.1f} | {t.max():.1f} | {c1[0] - c0[0]} | {c1[1] - c0[1]} | {(c1[4] - c0[4]) / steps:.1f} |")
            s.close()
    print()


def prefill_admission(P, torch, W, quick):
    print("## 4. Admitting a new request: alloc_reqid + step() until its prompt is backed (2048-token prompt, Llama-3-8B shape, 2 layers)\n")
    print("A request finishes (free_reqid), the next one arrives.  64 KiB page-groups: 64 page-groups per buffer, 256 in all.\n")
    print("| policy | admit mean us | max us | map calls per admission (critical path) | free_reqid mean us |")
    print("|---|---|---|---|---|")
    from paper_2405_04437_amd.binding import Vattn

    shape = W.LLAMA3_8B
    G, layers, B, prompt = 64 * KiB, 2, 8, 2048
    need = prompt * shape.token_bytes // G
    rounds = 10 if quick else 40
    for name, policy, flags, eager in (("unmap on free (synchronous)", P.POLICY_SYNC_UNMAP, 0, 0),
                                       ("deferred reclamation", P.POLICY_DEFERRED, 0, 0),
                                       ("deferred + background eager allocation", P.POLICY_DEFERRED, P.FLAG_BACKGROUND, need)):
        va = Vattn(layers, B, 4096, shape.num_q_heads, shape.num_kv_heads, shape.head_dim, 4 * need * 2 * layers * G, G,
                   policy=policy, flags=flags, lookahead_tokens=1, eager_page_groups=eager)
        seq = np.zeros(B, dtype=np.int64)
        # a resident request keeps the loop honest (step() always has someone to look at)
        r0 = va.alloc_reqid(); seq[r0] = 100
        assert va.step(seq) == 0
        times, frees, c0 = [], [], 0
        first = True
        for _ in range(rounds):
            va.sync()                      # the previous pass has had an iteration's time to finish
            t0 = time.perf_counter()
            r = va.alloc_reqid()
            seq[r] = prompt
            assert va.step(seq) == 0
            dt = (time.perf_counter() - t0) * 1e6
            if not first:
                times.append(dt)
            else:                          # the very first admission always maps from scratch: not counted
                c0 = va.step_counters()[0]
            first = False
            va.sync()
            seq[r] = 0
            t0 = time.perf_counter()
            assert va.free_reqid(r) == 0
            frees.append((time.perf_counter() - t0) * 1e6)
            assert va.step(seq) == 0       # an iteration without the request: the background pass prepares the next id
        c1 = va.step_counters()[0]
        t = np.array(times)
        print(f"| {name} | {t.mean():.1f} | {t.max():.1f} | {(c1 - c0) / (rounds - 1):.1f} | {np.mean(frees):.1f} |")
        va.destroy()
    print()


def fused_append(P, torch, W, quick):
    import time

    print("## 8. KV append as a launch of its own vs fused into the attention kernel\n")
    print("Wall time per call on the launch stream (calls queued back to back, one synchronisation at the end).\n")
    print("| path | separate append_kv + attention us | fused us | saved |")
    print("|---|---|---|---|")
    from paper_2405_04437_amd.runtime import KvSession

    def wall(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / iters

    # decode: Yi-6B shape, 32 requests x 8192 tokens, the newest token of each appended in the same call
    n, ctx = 32, 8192
    s, ids, shape, gen = _decode_session(P, torch, W, 2 * MiB, 0, n=n, ctx=ctx, layers=1)
    q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    kn = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    o = torch.empty_like(q)
    lens = [ctx] * n
    before = [ctx - 1] * n
    cu = list(range(n + 1))
    ws = s.workspace(lens)
    scale = W.softmax_scale(shape.head_dim)
    stream = s.stream

    def dec_sep():
        s.va.append_kv(0, stream, kn, kn, ids, cu, before)
        s.va.attn_decode(0, stream, q, o, ids, lens, scale, ws, ws.numel())

    a = wall(dec_sep, 300, 300)
    b = wall(lambda: s.va.attn_decode_append(0, stream, q, kn, kn, o, ids, lens, scale, ws, ws.numel()), 300, 300)
    print(f"| decode, 32 requests x 8192 tokens (Yi-6B shape) | {a:.1f} | {b:.1f} | {a - b:.1f} us ({100 * (a - b) / a:.1f} %) |")
    s.close()

    # prefill: the Llama-3-8B prefill batch of the benchmark (8 prompts, 105784 tokens)
    wl = W.config(2)
    shape = wl.shape
    kv_lens = [int(x) for x in wl.kv_lens]
    G = 2 * MiB
    per = (max(kv_lens) * shape.token_bytes + G - 1) // G * G
    s = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, len(kv_lens), max(kv_lens), per * 2 * len(kv_lens), 1, G)
    gen = torch.Generator(device="cuda"); gen.manual_seed(4)
    ids = [s.admit(L) for L in kv_lens]
    s.step()
    cu = [0]
    for L in kv_lens:
        cu.append(cu[-1] + L)
    tot = cu[-1]
    q = torch.empty((tot, shape.num_q_heads, shape.head_dim), device="cuda", dtype=torch.bfloat16)
    for a0 in range(0, tot, 16384):
        b0 = min(tot, a0 + 16384)
        q[a0:b0] = torch.randn((b0 - a0, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    kn = torch.randn((tot, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    o = torch.empty_like(q)
    zeros = [0] * len(kv_lens)
    stream = s.stream

    def pre_sep():
        s.va.append_kv(0, stream, kn, kn, ids, cu, zeros)
        s.va.attn_prefill(0, stream, q, o, ids, cu, kv_lens, scale)

    a = wall(pre_sep, 3 if quick else 6, 2)
    b = wall(lambda: s.va.attn_prefill_append(0, stream, q, kn, kn, o, ids, cu, kv_lens, scale), 3 if quick else 6, 2)
    print(f"| prefill, 8 prompts / {tot} tokens (Llama-3-8B shape) | {a:.0f} | {b:.0f} | {a - b:.0f} us ({100 * (a - b) / a:.1f} %) |")
    s.close()
    print()


def matrix_pipe(P):
    print("## 9. What the two roofs sustain: a register-only MFMA loop and a read-only stream\n")
    print("`v_mfma_f32_32x32x16_bf16`, operands in registers, no LDS or memory traffic in the timed loop; shader clock read")
    print("inside the kernel (cycle counter / 100 MHz counter).  N(0,1) is the value distribution of the attention workloads.\n")
    print("| operands | dense bf16 TFLOP/s | shader clock MHz | fraction of the 2.5 PFLOP/s peak |")
    print("|---|---|---|---|")
    for name, normal in (("all zero", False), ("N(0,1)", True)):
        best = max(P.mfma_microbench(normal, 200000) for _ in range(3))
        print(f"| {name} | {best[0]:.0f} | {best[1]:.0f} | {best[0] / 2500:.2f} |")
    print()
    print("The same loop with the side work of an attention inner loop added per matrix instruction (one operand read from LDS,")
    print("three fp32 multiply-adds, one exp2 - about what the prefill kernel issues per instruction): what each costs once the")
    print("power limit sets the clock, and what the whole mix sustains with nothing else in the way.\n")
    print("| per matrix instruction | N(0,1): TFLOP/s | MHz | all zero: TFLOP/s | MHz |")
    print("|---|---|---|---|---|")
    for name, kw in (("nothing else", {}), ("+ 16 B per lane from LDS as the A operand", {"lds_operand": True}), ("+ 3 fp32 FMA", {"fma3": True}),
                     ("+ 1 exp2", {"exp2": True}), ("+ all three", {"lds_operand": True, "fma3": True, "exp2": True})):
        n = max(P.mfma_microbench(True, 100000, **kw) for _ in range(2))
        z = max(P.mfma_microbench(False, 100000, **kw) for _ in range(2))
        print(f"| {name} | {n[0]:.0f} | {n[1]:.0f} | {z[0]:.0f} | {z[1]:.0f} |")
    print()
    print("And what HBM delivers to a kernel that only reads: one workgroup of four waves per CU, each a contiguous share,")
    print("16-byte non-temporal loads, 16 per lane in flight (the decode kernel's launch shape without its arithmetic).\n")
    print("| buffer | GB/s | fraction of the 8 TB/s peak |")
    print("|---|---|---|")
    for gib in (1, 4, 16):
        g = P.stream_microbench(gib << 30)
        print(f"| {gib} GiB | {g:.0f} | {g / 8000:.2f} |")
    print()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", type=int, default=0, help="run only the section with this number")
    ap.add_argument("--quick", action="store_true")
    args = ap.parse_args()
    import torch

    if not torch.cuda.is_available():
        print("vmm_report.py needs a GPU", file=sys.stderr)
        return 1
    import paper_2405_04437_amd as P
    import workloads as W

    torch.cuda.set_stream(torch.cuda.Stream())
    print(f"# Memory-manager measurements on {torch.cuda.get_device_name(0)}\n")
    print("Command: `python vmm_report.py" + (" --quick" if args.quick else "") + (f" --only {args.only}" if args.only else "") + "`\n")
    sections = {1: lambda: api_latency(P, args.quick), 2: lambda: page_size_effect(P, torch, W, args.quick),
                3: lambda: latency_hiding(P, torch, W, args.quick), 4: lambda: prefill_admission(P, torch, W, args.quick),
                5: lambda: paged_overhead(P, torch, W, args.quick), 6: lambda: slicing_effect(P, torch, W, args.quick),
                7: lambda: fragmentation(P, W, args.quick), 8: lambda: fused_append(P, torch, W, args.quick),
                9: lambda: matrix_pipe(P)}
    for num, fn in sections.items():
        if args.only in (0, num):
            fn()
    return 0


if __name__ == "__main__":
    sys.exit(main())
