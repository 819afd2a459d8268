#!/usr/bin/env python3
"""Benchmark of the contiguous-KV attention hot path on one MI355X.

Headline workload (N=1): BASELINE config 2, "Yi-6B-shaped decode" - 64 requests, 32 query heads,
4 KV heads, head_dim 128, bf16, contexts U[1024,16384], 32 decoder layers (44 GB of KV).  A step is one
serving iteration of Algorithm 1 in which every request grows by one token:
    step()  ->  for each of the 32 layers: attn_decode_append (the new K/V row is written by the
                split-K kernel that reads the cache, then the reduce kernel)  ->  stream synchronise
i.e. one pass over all rows of the hot path at the model's depth.  The KV grows on the library's helper
thread with a 64-token look-ahead (Sec. 6.1); --sync-maps maps inside step() instead.  `value` is
algorithmic KV bytes moved per second over the whole step (inputs resident in HBM); `roofline` prices
the dominant kernel (split-K decode) alone, timed with HIP events the library records around every
launch on the launch stream; `roofline.prefill` (repeated as the top-level `roofline_prefill`) prices the
prefill kernel on config 3 the same way, the second half of the two-part metric.

`also` carries the other configurations: config 3 (prefill), config 4 as ONE mixed serving iteration
(128 decodes + a 2048-token chunk appended at 8192 + 10 % of the requests leaving and arriving, memory
management overlapped with the previous iteration and done by the helper thread: look-ahead, deferred
reclamation, eager allocation - Sec. 6.1), and config 5 (131072-token prefill, then decode).
`cpu_baseline` is the CPU oracle timed on the same decode batch; `cpu_baseline.prefill` times it on
>= 512 sampled query rows of each prefill workload and extrapolates linearly to the whole workload.

Synthetic data: N(0,1) bf16 Q/K/V drawn on the device from a seeded generator; context lengths from
workloads.config().  Nothing is read from disk except the measured-traffic file under profiles/
(rocprofv3 counter results, stamped with the command they were measured with).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MiB = 1024 * 1024


def _decode_bytes(shape, kv_lens):
    """Algorithmic bytes of one decode layer-step: every K and V byte once, Q read, O written."""
    per_tok = 2 * shape.num_kv_heads * shape.head_dim * 2
    qo = 2 * shape.num_q_heads * shape.head_dim * 2
    return sum(int(L) * per_tok + qo for L in kv_lens)


def _visible_pairs(q_lens, kv_lens):
    tot = 0
    for ql, kl in zip(q_lens, kv_lens):
        off = kl - ql
        tot += ql * off + ql * (ql + 1) // 2
    return tot


def _prefill_flops(shape, q_lens, kv_lens):
    """Causal-only flops: 4*Hq*D per (query row, visible key) pair."""
    return 4 * shape.num_q_heads * shape.head_dim * _visible_pairs(q_lens, kv_lens)


def _ok(rc):
    if rc != 0:
        from paper_2405_04437_amd import last_error
        raise RuntimeError("libvattn call failed: " + last_error())


def _randn_bf16(torch, gen, shape):
    if gen is None:                                  # all-zero operands: the chip keeps its full clock (see run_prefill)
        return torch.zeros(shape, device="cuda", dtype=torch.bfloat16)
    return torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)


def _fill_contexts(sess, torch, gen, shape, kv_lens, layers, keep_host=False):
    """Admit the requests, back them with step() and write N(0,1) K/V through append_kv."""
    ids = [sess.admit(int(L)) for L in kv_lens]
    sess.step()
    host = []
    for r, L in zip(ids, kv_lens):
        done = 0
        ks, vs = [], []
        while done < L:
            n = min(8192, L - done)
            k = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
            v = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
            for layer in range(layers):
                sess.append(layer, k, v, [r], [0, n], [done])
            if keep_host:
                ks.append(k.cpu()); vs.append(v.cpu())
            done += n
        if keep_host:
            host.append((torch.cat(ks), torch.cat(vs)))
    torch.cuda.synchronize()
    return ids, host


def run_decode(args, torch, W, wl, steps, warmup, layers=2, with_oracle=True, whole_model=False, background=False):
    """Decode steps.  whole_model=False: one layer's attention per step (the layer rotates) and a stream
    synchronisation after it.  whole_model=True: a serving iteration - step() once, then the fused
    append + attention of every one of `layers` layers, then the synchronisation (Algorithm 1)."""
    from paper_2405_04437_amd import FLAG_BACKGROUND, POLICY_DEFERRED
    from paper_2405_04437_amd.runtime import KvSession, tensor_to_bits, tensor_to_f32
    import numpy as np

    shape = wl.shape
    n = sum(1 for q in wl.q_lens if q == 1)
    kv_lens = [int(x) for x in wl.kv_lens[:n]]
    ksteps = max(20, steps // 8) if whole_model else steps    # steps of the second, event-timed pass
    # A freshly started process shows one 30-40 ms device stall within its first ~50 ms of sustained launches: besides
    # the --warmup steps the caller asks for, a whole-model run first keeps the GPU busy for ~100 ms, untimed.
    settle = 16 if whole_model else 0
    total_steps = steps + ksteps + warmup + settle + 2
    max_ctx = max(kv_lens) + total_steps + 8 + 64
    G = 2 * MiB
    headroom = n // 4 + 4
    lookahead = 64 if background else 0
    # the page-groups these requests can reach by the last step (look-ahead included), and a few spare rows
    rows = sum((int(L + total_steps + 8 + lookahead) * shape.token_bytes + G - 1) // G for L in kv_lens) + 8
    budget = rows * G * 2 * layers
    sess = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + headroom, max_ctx, budget, layers, G,
                     POLICY_DEFERRED, flags=FLAG_BACKGROUND if background else 0, lookahead_tokens=lookahead)
    gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    ids, host = _fill_contexts(sess, torch, gen, shape, kv_lens, layers, keep_host=with_oracle)
    for r, L in zip(ids, kv_lens):
        sess.seq_lens[r] = L
    scale = W.softmax_scale(shape.head_dim)
    q = _randn_bf16(torch, gen, (n, shape.num_q_heads, shape.head_dim))
    knew = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
    vnew = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
    o = torch.empty_like(q)
    lens = np.array(kv_lens, dtype=np.int64)
    ids = np.array(ids, dtype=np.int32)
    seq = np.zeros(sess.B, dtype=np.int64)      # cache_seq_len of Algorithm 1, indexed by reqId
    ws = sess.workspace([int(L) + total_steps for L in lens])
    cu = np.arange(n + 1, dtype=np.int32)
    per_tok = 2 * shape.num_kv_heads * shape.head_dim * 2
    qo_bytes = n * 2 * shape.num_q_heads * shape.head_dim * 2
    va, stream = sess.va, sess.stream
    torch_stream = torch.cuda.current_stream()

    every = {"bytes": 0, "launches": 0}     # over every decode launch of this run, warm-up included (for counter runs)

    def one_step(i):
        seq[ids] = lens + 1
        _ok(va.step(seq))
        every["bytes"] += (int(lens.sum() + n) * per_tok + qo_bytes) * (layers if whole_model else 1)
        every["launches"] += layers if whole_model else 1
        if whole_model:                   # every layer: the new K/V row rides in that layer's decode kernel
            for layer in range(layers):
                _ok(va.attn_decode_append(layer, stream, q, knew, vnew, o, ids, lens + 1, scale, ws, ws.numel()))
        else:
            att = i % layers              # the layer attended to in this step; its append rides in the decode kernel
            _ok(va.attn_decode_append(att, stream, q, knew, vnew, o, ids, lens + 1, scale, ws, ws.numel()))
            for layer in range(layers):   # the other layers' appends are independent of it and queue up behind
                if layer != att:
                    _ok(va.append_kv(layer, stream, knew, vnew, ids, cu, lens))
        lens[:] += 1
        # iteration boundary of the serving loop (Algorithm 1): the framework needs this iteration's
        # output on the host before it can schedule the next one
        torch_stream.synchronize()

    launches_per_step = layers if whole_model else 1

    def step_bytes():
        return (int(lens.sum()) * per_tok + qo_bytes) * launches_per_step

    for i in range(settle + warmup):
        one_step(i)
    torch.cuda.synchronize()
    map0 = sess.va.counters()
    bytes_total = 0
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(warmup + i)
        bytes_total += step_bytes()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    map1 = sess.va.counters()
    # second pass, same steps again, with the library's per-launch HIP events switched on: the average
    # launch duration of the split-K kernel (the event records perturb the whole-step time, so the
    # two are measured separately)
    sess.va.set_timing(True)
    sess.va.kernel_time(0); sess.va.kernel_time(2); sess.va.kernel_time(3)
    kbytes = 0
    k_ms = r_ms = 0.0
    k_n = r_n = 0
    per_step_us = []                          # average split-K launch of each event-timed step
    for i in range(ksteps):
        one_step(warmup + steps + i)
        kbytes += step_bytes()
        a_ms, a_n = sess.va.kernel_time(0)
        b_ms, b_n = sess.va.kernel_time(2)
        k_ms += a_ms; k_n += a_n; r_ms += b_ms; r_n += b_n
        per_step_us.append(a_ms / max(a_n, 1) * 1e3)
    torch.cuda.synchronize()
    sess.va.set_timing(False)
    per_step_us.sort()
    kbytes_per_launch = kbytes / max(k_n, 1)
    ms_per_step = (t1 - t0) * 1e3 / steps
    bytes_per_step = bytes_total / steps
    res = {
        "ms_per_step": ms_per_step,
        "gbs_step": bytes_per_step / (ms_per_step * 1e6),
        "kernel_ms": k_ms / max(k_n, 1),
        "reduce_ms": r_ms / max(r_n, 1),
        "gbs_kernel": kbytes_per_launch / (k_ms / max(k_n, 1) * 1e6),
        "kernel_us_median_over_steps": per_step_us[len(per_step_us) // 2], "kernel_us_min_over_steps": per_step_us[0],
        "event_timed_steps": ksteps, "event_timed_launches": k_n,
        "bytes_per_step": bytes_per_step,
        "kbytes_per_launch": kbytes_per_launch,
        "tokens_in_batch": int(lens.sum()),
        "bytes_per_launch_over_all_launches": every["bytes"] / max(every["launches"], 1), "all_launches": every["launches"],
        "layers": layers, "decode_launches_per_step": launches_per_step, "settle_steps_before_warmup": settle,
        "map_calls_in_timed_region": map1[0] - map0[0],
        "map_us_in_timed_region": map1[2] - map0[2],
        "unmap_calls_in_timed_region": map1[1] - map0[1],
    }
    if with_oracle:
        # CPU oracle on the same batch as the last timed step (layer = last used layer).
        from oracle import attention as OA

        last_layer = layers - 1 if whole_model else (warmup + steps + ksteps - 1) % layers
        torch.cuda.synchronize()
        qb = tensor_to_bits(q)
        kb_new, vb_new = tensor_to_bits(knew), tensor_to_bits(vnew)
        ks, vs = [], []
        grown = int(lens[0]) - kv_lens[0]
        for r in range(n):
            k0, v0 = host[r]
            ks.append(np.concatenate([tensor_to_bits(k0)] + [kb_new[r:r + 1]] * grown))
            vs.append(np.concatenate([tensor_to_bits(v0)] + [vb_new[r:r + 1]] * grown))
        reps = 4   # ~30 core-seconds of oracle work on a 16-core host
        t0 = time.perf_counter()
        for _ in range(reps):
            want = OA.attention_batch(qb, np.arange(n + 1), ks, vs, scale)
        dt = (time.perf_counter() - t0) / reps
        got = tensor_to_f32(o)
        err = float(np.abs(got - want).max())
        rel = float((np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max())
        res["cpu_baseline"] = {
            "value": step_bytes() / launches_per_step / dt / 1e9, "unit": "GB/s", "cores": OA.num_threads(), "kind": "oracle",
            "sample": f"the full decode batch of the last timed step ({n} requests, {int(lens.sum())} tokens, layer {last_layer}), {reps} times: {dt:.2f} s each",
            "gpu_vs_oracle_max_abs": err, "gpu_vs_oracle_row_rel": rel,
        }
    sess.close()
    return res


def run_mixed(args, torch, W, wl, steps, warmup):
    """Config 4 as one serving iteration per step: 128 decode requests grow by a token, a 2048-token chunk
    is appended to a request at 8192 (its K/V rows written by the prefill kernel itself), and 10 % of the
    decode requests leave while as many arrive (their contexts written in place).  The loop is the
    overlapped one of Sec. 6.1: while the GPU runs iteration i-1 the host retires and admits requests and
    calls step() for iteration i; the helper thread maps the look-ahead, tops up the reqId that will be
    handed out next and reclaims when the pool runs low.  A request is freed one window after it left the
    batch, i.e. when no kernel can still read it."""
    from paper_2405_04437_amd import FLAG_BACKGROUND, POLICY_DEFERRED
    from paper_2405_04437_amd.runtime import KvSession
    import numpy as np

    shape = wl.shape
    n = sum(1 for q in wl.q_lens if q == 1)
    kv_lens = [int(x) for x in wl.kv_lens[:n]]
    chunk_q = int(wl.q_lens[n]); chunk_ctx = int(wl.kv_lens[n])       # 2048 rows ending at 10240
    lo, hi = wl.extra["ctx_range"]
    k_churn = max(1, int(round(wl.extra["churn_fraction"] * n)))
    ksteps = max(4, steps // 4)
    total_steps = 2 * steps + ksteps + warmup + 160 + 8
    max_ctx = hi + total_steps + 8 + 64
    G = 2 * MiB
    tok = shape.token_bytes
    rows_of = lambda L: (int(L) * tok + G - 1) // G
    headroom = 3 * k_churn + 4                     # ids retired but not yet freed, ids being admitted, spares
    B = n + 1 + headroom
    # Pool: every reqId can be backed at full length (22 GB here, one layer).  Under deferred reclamation a reqId keeps
    # the most page-groups any of its past requests needed, so a pool sized for the batch's AVERAGE context runs dry
    # within a few iterations; the threshold below makes the helper thread give inactive ids' pages back when less
    # than 5 % of the pool is free, which this sizing reaches only if the batch is unusually long.
    pool_rows = B * rows_of(max_ctx)
    sess = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, B, max_ctx, pool_rows * G * 2, 1, G,
                     POLICY_DEFERRED, flags=FLAG_BACKGROUND, lookahead_tokens=64, eager_page_groups=rows_of(hi),
                     reclaim_threshold_page_groups=2 * (pool_rows // 20))
    gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    ids, _ = _fill_contexts(sess, torch, gen, shape, kv_lens + [chunk_ctx - chunk_q], 1)
    chunk_id = ids.pop()
    scale = W.softmax_scale(shape.head_dim)
    q = _randn_bf16(torch, gen, (n, shape.num_q_heads, shape.head_dim))
    knew = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
    vnew = _randn_bf16(torch, gen, (n, shape.num_kv_heads, shape.head_dim))
    o = torch.empty_like(q)
    qc = _randn_bf16(torch, gen, (chunk_q, shape.num_q_heads, shape.head_dim))
    kc = _randn_bf16(torch, gen, (chunk_q, shape.num_kv_heads, shape.head_dim))
    vc = _randn_bf16(torch, gen, (chunk_q, shape.num_kv_heads, shape.head_dim))
    oc = torch.empty_like(qc)
    # source rows for the contexts of arriving requests (their earlier prefill's KV), packed
    kbig = _randn_bf16(torch, gen, (k_churn * (hi + 512), shape.num_kv_heads, shape.head_dim))
    vbig = _randn_bf16(torch, gen, (k_churn * (hi + 512), shape.num_kv_heads, shape.head_dim))
    lens = np.array(kv_lens, dtype=np.int64)
    ids = np.array(ids, dtype=np.int32)
    seq = np.zeros(B, dtype=np.int64)
    ws = sess.workspace([hi + total_steps] * n)
    rng = np.random.default_rng(wl.seed)
    va, stream = sess.va, sess.stream
    torch_stream = torch.cuda.current_stream()
    chunk_ids = np.array([chunk_id], dtype=np.int32)
    chunk_cu = np.array([0, chunk_q], dtype=np.int32)
    chunk_kv = np.array([chunk_ctx], dtype=np.int64)
    retired = []                                   # reqIds that left the batch in the previous window
    stat = {"arrival_map_demand": 0, "host_window_us": 0.0, "decode_bytes": 0}
    every = {"bytes": 0, "launches": 0}           # over every decode launch of this run (for counter runs)

    def one_step(i, launch=True):
        t_host = time.perf_counter()
        # ---- host window: the GPU is still running iteration i-1 -------------------------------------------
        for r in retired:                          # left the batch before iteration i-1 was launched: nothing reads them
            seq[r] = 0
            _ok(va.free_reqid(int(r)))
        retired.clear()
        slots = rng.choice(n, size=k_churn, replace=False)
        for s in slots:                            # these are part of the running iteration i-1: free them next time
            retired.append(int(ids[s]))
            lens[s] = int(rng.integers(lo, hi, endpoint=True))
            ids[s] = va.alloc_reqid()
            assert ids[s] >= 0
        # bookkeeping only: what step() will have to map for the newcomers (everything else it maps is growth of
        # running requests, which the look-ahead of the previous pass should already have covered)
        for s in slots:
            stat["arrival_map_demand"] += 2 * max(0, rows_of(lens[s] + 1) - va.query(int(ids[s]))[1])
        for r in retired:
            seq[r] = 0                             # out of the batch: step() needs nothing for them (still active until freed)
        seq[ids] = lens + 1
        seq[chunk_id] = chunk_ctx
        _ok(va.step(seq))
        stat["host_window_us"] += (time.perf_counter() - t_host) * 1e6
        acu = np.zeros(k_churn + 1, dtype=np.int32)
        acu[1:] = np.cumsum(lens[slots])
        rows_new = int(acu[-1])
        if not launch:                             # ageing the allocator: the memory management of an iteration without its kernels
            lens[:] += 1
            return rows_new
        # ---- iteration boundary: iteration i-1's output is needed before iteration i is launched -------------
        torch_stream.synchronize()
        _ok(va.append_kv(0, stream, kbig[:rows_new], vbig[:rows_new], ids[slots], acu, np.zeros(k_churn, dtype=np.int64)))
        _ok(va.attn_prefill_append(0, stream, qc, kc, vc, oc, chunk_ids, chunk_cu, chunk_kv, scale))
        _ok(va.attn_decode_append(0, stream, q, knew, vnew, o, ids, lens + 1, scale, ws, ws.numel()))
        lens[:] += 1
        stat["decode_bytes"] += _decode_bytes(shape, lens)
        every["bytes"] += _decode_bytes(shape, lens); every["launches"] += 1
        return rows_new

    def counters():
        a = va.counters(); b = va.step_counters()
        return {"map": a[0], "unmap": a[1], "map_us": a[2], "unmap_us": a[3], "sync_map": b[0], "bg_map": b[1],
                "step_us": b[2], "bg_us": b[3], "wait_us": b[4]}

    def timed_region(first, count):
        for k in stat:
            stat[k] = 0
        c0 = counters()
        t0 = time.perf_counter()
        for i in range(count):
            one_step(first + i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / count
        c1 = counters()
        return ms, {k: c1[k] - c0[k] for k in c0}, dict(stat)

    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()
    # 1. cold: the first iterations after start-up, when most arriving requests are longer than anything their
    #    reqId has held before, so their contexts still have to be mapped
    cold_ms, cold_d, cold_stat = timed_region(warmup, steps)
    # 2. the allocator is aged to its steady state (the memory management of `age` more iterations, no kernels):
    #    under deferred reclamation every reqId ends up holding what its longest request needed
    age = 160
    for i in range(age):
        one_step(warmup + steps + i, launch=False)
    va.sync()
    for s0 in range(0, n, k_churn):               # the requests admitted while ageing get their contexts written now
        sl = np.arange(s0, min(n, s0 + k_churn))
        acu = np.zeros(len(sl) + 1, dtype=np.int32)
        acu[1:] = np.cumsum(lens[sl])
        _ok(va.append_kv(0, stream, kbig[:int(acu[-1])], vbig[:int(acu[-1])], ids[sl], acu, np.zeros(len(sl), dtype=np.int64)))
    for i in range(3):
        one_step(warmup + steps + age + i)
    torch.cuda.synchronize()
    # 3. steady state, timed
    ms_per_step, d, timed = timed_region(warmup + steps + age + 3, steps)
    timed = dict(stat)
    # second pass with per-launch HIP events: what the GPU spends inside the kernels of one iteration
    va.set_timing(True)
    for w in range(4):
        va.kernel_time(w)
    dbytes0 = stat["decode_bytes"]
    arr_rows = 0
    for i in range(ksteps):
        arr_rows += one_step(warmup + 2 * steps + 163 + i)
    torch.cuda.synchronize()
    kt = [va.kernel_time(w) for w in range(4)]     # split-K, prefill, reduce, append
    va.set_timing(False)
    dec_ms, pre_ms, red_ms, app_ms = [t / max(c, 1) for t, c in kt]
    app_ms_step = kt[3][0] / ksteps
    dbytes = (stat["decode_bytes"] - dbytes0) / ksteps
    chunk_flops = _prefill_flops(shape, [chunk_q], [chunk_ctx])
    sum_kernels = dec_ms + red_ms + pre_ms + app_ms_step
    held_rows = sum(va.query(int(r))[1] for r in range(B))
    needed_rows = int(sum(rows_of(L) for L in lens)) + rows_of(chunk_ctx)
    sess.close()
    return {
        "ms_per_step": ms_per_step, "sum_of_kernel_ms": sum_kernels, "step_over_kernels": ms_per_step / sum_kernels,
        "kernel_ms": {"decode_splitk": dec_ms, "decode_reduce": red_ms, "prefill_chunk": pre_ms,
                      "arrivals_kv_write_per_step": app_ms_step},
        "decode_gbs_kernel": dbytes / (dec_ms * 1e6), "decode_frac_of_hbm_peak": dbytes / (dec_ms * 1e6) / HBM_PEAK_GBS,
        "decode_bytes_per_launch": dbytes,
        "decode_bytes_per_launch_over_all_launches": every["bytes"] / max(every["launches"], 1), "all_decode_launches": every["launches"],
        "chunk_flops_per_launch": chunk_flops,
        "chunk_tflops_kernel": chunk_flops / (pre_ms * 1e9), "chunk_frac_of_bf16_mfma_peak": chunk_flops / (pre_ms * 1e9) / MFMA_BF16_PEAK_TFLOPS,
        "arrivals_kv_write_gbs": 2 * 2 * (arr_rows / ksteps) * tok / (app_ms_step * 1e6) if app_ms_step > 0 else None,
        "requests_leaving_and_arriving_per_step": k_churn,
        "host_window_us_per_step": timed["host_window_us"] / steps,
        "step_call_us_per_step": d["step_us"] / steps,
        "map_calls_per_step": {"inside_step_total": d["sync_map"] / steps,
                               "inside_step_for_arrivals": timed["arrival_map_demand"] / steps,
                               "inside_step_for_running_requests": (d["sync_map"] - timed["arrival_map_demand"]) / steps,
                               "by_background_passes": d["bg_map"] / steps},
        "unmap_calls_per_step": d["unmap"] / steps,
        "allocator_state": f"steady: aged by {age} iterations of arrivals and departures before timing",
        "page_group_rows_mapped_vs_needed": [held_rows, needed_rows],
        "cold_start": {"what": f"the first {steps} iterations after start-up ({warmup} warm-up iterations before them)",
                       "ms_per_step": cold_ms, "host_window_us_per_step": cold_stat["host_window_us"] / steps,
                       "map_calls_per_step": {"inside_step_total": cold_d["sync_map"] / steps,
                                              "inside_step_for_arrivals": cold_stat["arrival_map_demand"] / steps,
                                              "inside_step_for_running_requests": (cold_d["sync_map"] - cold_stat["arrival_map_demand"]) / steps,
                                              "by_background_passes": cold_d["bg_map"] / steps},
                       "waited_for_pass_us_per_step": cold_d["wait_us"] / steps},
        "background_pass_us_per_step": d["bg_us"] / steps, "waited_for_pass_us_per_step": d["wait_us"] / steps,
        "pool_page_groups": 2 * pool_rows,
        "memory_management": "deferred reclamation + helper thread: 64-token look-ahead, eager allocation of one full-length reqId, "
                             "threshold reclamation; free/alloc/step() overlapped with the previous iteration",
    }


def run_prefill(args, torch, W, wl, iters, warmup, oracle_rows=0, name="", zero_operands=False):
    """Prefill launches of the workload's requests with q_len > 1, timed one by one.  oracle_rows > 0: the CPU
    oracle evaluates that many sampled query rows (spread over the requests), is timed, and the GPU output is
    compared with it on those rows.  zero_operands: Q, K and V are all zeros - the same instruction stream without
    the operand toggling that makes the chip lower its clock to hold its power limit, i.e. how well the kernel
    keeps the matrix pipes busy at full clock (not a throughput claim)."""
    from paper_2405_04437_amd.runtime import KvSession, tensor_to_bits, tensor_to_f32
    import numpy as np

    shape = wl.shape
    idx = [i for i, ql in enumerate(wl.q_lens) if ql > 1]
    q_lens = [int(wl.q_lens[i]) for i in idx]
    kv_lens = [int(wl.kv_lens[i]) for i in idx]
    n = len(idx)
    G = 2 * MiB
    max_ctx = max(kv_lens)
    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    sess = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n, max_ctx, per_req * 2 * n, 1, G)
    gen = None
    if not zero_operands:
        gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    ids, host = _fill_contexts(sess, torch, gen, shape, kv_lens, 1, keep_host=oracle_rows > 0)
    cu = [0]
    for ql in q_lens:
        cu.append(cu[-1] + ql)
    q = torch.empty((cu[-1], shape.num_q_heads, shape.head_dim), device="cuda", dtype=torch.bfloat16)
    for a in range(0, cu[-1], 16384):
        b = min(cu[-1], a + 16384)
        q[a:b] = _randn_bf16(torch, gen, (b - a, shape.num_q_heads, shape.head_dim))
    o = torch.empty_like(q)
    scale = W.softmax_scale(shape.head_dim)
    for _ in range(warmup):
        sess.prefill(0, q, ids, cu, kv_lens, scale, out=o)
    torch.cuda.synchronize()
    # Every launch is timed by itself (HIP events on its dispatch) and the MEDIAN launch is reported: a freshly
    # started process shows an occasional launch that is stalled for several milliseconds.
    sess.va.set_timing(True); sess.va.kernel_time(1)
    per_launch, walls = [], []
    for _ in range(iters):
        t0 = time.perf_counter()
        sess.prefill(0, q, ids, cu, kv_lens, scale, out=o)
        torch.cuda.synchronize()
        walls.append((time.perf_counter() - t0) * 1e3)
        k_ms, k_n = sess.va.kernel_time(1)
        per_launch.append(k_ms / max(k_n, 1))
    sess.va.set_timing(False)
    order = sorted(range(iters), key=lambda i: per_launch[i])
    mid = order[(iters - 1) // 2]
    flops = _prefill_flops(shape, q_lens, kv_lens)
    ms, kms = walls[mid], per_launch[mid]
    res = {"ms_per_call": ms, "kernel_ms": kms, "tflops_call": flops / (ms * 1e9), "tflops_kernel": flops / (kms * 1e9),
           "frac_of_mfma_peak": flops / (kms * 1e9) / MFMA_BF16_PEAK_TFLOPS, "flops": flops, "q_tokens": cu[-1],
           "kernel_ms_per_launch": [round(x, 4) for x in per_launch]}
    if oracle_rows > 0:
        from oracle import attention as OA

        per_req_rows = -(-oracle_rows // n)
        pairs = 0
        secs = 0.0
        err = rel = 0.0
        nrows = 0
        for r in range(n):
            off = kv_lens[r] - q_lens[r]
            edges = [x for x in (384, 385, q_lens[r] - 384, 64 - off % 64, 1024 - off % 1024) if 0 < x < q_lens[r]]
            rows = W.sample_rows(q_lens[r], per_req_rows, seed=wl.seed + r, boundaries=edges)
            sel = torch.from_numpy(rows.astype(np.int64)).cuda()
            qr = q[cu[r]:cu[r + 1]]
            kb, vb = tensor_to_bits(host[r][0]), tensor_to_bits(host[r][1])
            # each sampled row as a one-row chunk whose context ends at that row (the same causal definition,
            # without copying all of Q to the host); the rows of a request run in one oracle call
            qb = np.zeros((q_lens[r], shape.num_q_heads, shape.head_dim), dtype=np.uint16)
            qb[rows] = tensor_to_bits(qr[sel])
            t0 = time.perf_counter()
            want = OA.attention_request(qb, kb, vb, scale, rows=rows)
            secs += time.perf_counter() - t0
            got = tensor_to_f32(o[cu[r]:cu[r + 1]][sel])
            e = np.abs(got - want).max(axis=-1)
            err = max(err, float(e.max())); rel = max(rel, float((e / np.abs(want).max(axis=-1)).max()))
            pairs += int(sum(int(x) + off + 1 for x in rows))
            nrows += len(rows)
        full_pairs = _visible_pairs(q_lens, kv_lens)
        sample_flops = 4 * shape.num_q_heads * shape.head_dim * pairs
        res["cpu_baseline"] = {
            "value": sample_flops / secs / 1e12, "unit": "TFLOP/s", "cores": OA.num_threads(), "kind": "oracle",
            "sample": f"{nrows} sampled query rows of {name} (all {shape.num_q_heads} heads each; first, last, tile- and page-edge "
                      f"rows and uniformly drawn ones), {pairs} visible (query, key) pairs",
            "sample_seconds": secs,
            "extrapolated_full_workload_seconds": secs * full_pairs / pairs,
            "extrapolation": "linear in visible (query, key) pairs: sample_seconds x all pairs / sampled pairs",
            "gpu_vs_oracle_max_abs": err, "gpu_vs_oracle_row_rel": rel,
        }
    sess.close()
    return res


def _measured_traffic(name, steps, warmup):
    """HBM bytes per launch from the committed rocprofv3 counter summary - only when this run uses the step
    counts the counters were collected with (the batch, and with it the bytes per launch, grows with every step)."""
    p = os.path.join(ROOT, "profiles", "measured_traffic.json")
    try:
        with open(p) as f:
            d = json.load(f)
    except Exception:
        return None, None
    e = d.get(name)
    if not e:
        return None, None
    stamp = {"command": e.get("command"), "steps": e.get("steps"), "warmup": e.get("warmup")}
    if e.get("steps") is not None and (e.get("steps") != steps or e.get("warmup") != warmup):
        return None, dict(stamp, note="not reported: this run's --steps/--warmup differ from the profiled command's")
    return e, stamp


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps; the first ~50 ms of sustained load on a fresh process contain a one-off "
                         "30-40 ms device stall (seen between two back-to-back launches), so keep this >= 5 "
                         "whole-model steps")
    ap.add_argument("--only", choices=["all", "decode", "prefill", "mixed", "c5", "copy"], default="all")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="decoder layers per decode step (0 = the model's depth)")
    ap.add_argument("--sync-maps", action="store_true", help="grow the KV inside step() instead of on the helper thread")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards by request / KV head with no exchange "
              "step); run with --gpus 1", file=sys.stderr)
        return 2
    import torch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP path has no CPU fallback", file=sys.stderr)
        return 1
    import workloads as W

    # A stream of its own: on the legacy default stream HIP serialises host-side copies with the device.
    torch.cuda.set_stream(torch.cuda.Stream())

    out = {"metric": "decode attn HBM GB/s (% of peak) + prefill attn TFLOP/s (% MFMA peak)", "unit": "GB/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": {}}
    also = {}
    oracle_on = not args.no_cpu_baseline
    if args.only == "copy":
        # Calibration for the HBM-traffic counters: a plain device copy of known size (1 GiB read + 1 GiB
        # written per launch), so that FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes.
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch device copy", "bytes_read_per_launch": n, "bytes_written_per_launch": n, "launches": 5}))
        return 0
    if args.only in ("all", "decode"):
        wl = W.config(1)
        depth = args.layers or wl.shape.num_layers
        r = run_decode(args, torch, W, wl, args.steps, args.warmup, layers=depth, with_oracle=oracle_on,
                       whole_model=True, background=not args.sync_maps)
        out["config"] = {"workload": f"C2 Yi-6B-shaped decode at the model's depth: 64 requests, Hq=32 H=4 D=128, ctx U[1024,16384], "
                                     f"{depth} layers (one split-K + one reduce launch per layer and step), one token per request per step "
                                     "(step(), then per layer: K/V append fused into split-K decode, reduce), 2 MiB page-groups",
                         "kv_growth": "step() on the caller's thread" if args.sync_maps else "helper thread, 64-token look-ahead"}
        out["value"] = r["gbs_step"]
        out["ms_per_step"] = r["ms_per_step"]
        out["pct_of_hbm_peak"] = 100.0 * r["gbs_step"] / HBM_PEAK_GBS
        traffic, stamp = _measured_traffic("decode_splitk_C2", args.steps, args.warmup)
        out["roofline"] = {"kernel": "decode_splitk_kernel<128>", "bound": "hbm", "achieved": r["gbs_kernel"],
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": r["gbs_kernel"] / HBM_PEAK_GBS,
                           "avg_launch_ms": r["kernel_ms"], "median_launch_ms_over_steps": r["kernel_us_median_over_steps"] / 1e3,
                           "min_launch_ms_over_steps": r["kernel_us_min_over_steps"] / 1e3, "timed_launches": r["event_timed_launches"],
                           "algorithmic_bytes_per_launch": r["kbytes_per_launch"],
                           "traffic": (traffic or {}).get("total_bytes"),
                           "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                           "traffic_measured_with": stamp, "traffic_detail": traffic}
        if "cpu_baseline" in r:
            out["cpu_baseline"] = r.pop("cpu_baseline")
        out["decode_detail"] = {k: r[k] for k in ("reduce_ms", "tokens_in_batch", "settle_steps_before_warmup", "bytes_per_launch_over_all_launches", "all_launches", "map_calls_in_timed_region",
                                                  "map_us_in_timed_region", "unmap_calls_in_timed_region")}
        # what a read-only kernel of the same launch shape gets out of HBM (4 GiB, best of three launches)
        import paper_2405_04437_amd as P
        stream = P.stream_microbench(4 << 30)
        out["roofline"]["sustained_read_gbs"] = stream
        out["roofline"]["frac_of_sustained_read"] = r["gbs_kernel"] / stream
        if args.only == "all":
            # the same batch with a host synchronisation after every single layer's attention: the
            # cost of the per-iteration host work when nothing amortises it
            r1 = run_decode(args, torch, W, wl, 400, 300, layers=2, with_oracle=False)
            also["C2_one_layer_per_sync"] = {"gbs_step": r1["gbs_step"], "ms_per_step": r1["ms_per_step"],
                                             "gbs_kernel": r1["gbs_kernel"], "kernel_ms": r1["kernel_ms"]}
    prefill_cpu = {}
    if args.only in ("all", "prefill"):
        wl3 = W.config(2)
        p = run_prefill(args, torch, W, wl3, iters=7, warmup=2, oracle_rows=512 if oracle_on else 0,
                        name="C3 (8 prompts U[4096,32768])")
        traffic, stamp = _measured_traffic("prefill_C3", None, None)
        also["C3_llama3_8b_prefill"] = {"tflops": p["tflops_call"], "kernel_tflops": p["tflops_kernel"],
                                        "frac_of_bf16_mfma_peak": p["frac_of_mfma_peak"],
                                        "ms": p["ms_per_call"],
                                        "kernel_ms": p["kernel_ms"], "kernel_ms_per_launch": p["kernel_ms_per_launch"], "q_tokens": p["q_tokens"],
                                        "flop_convention": "causal only: 4*Hq*D per visible (query,key) pair"}
        out["roofline_prefill"] = {"kernel": "prefill_kernel<128>", "workload": "C3 Llama-3-8B-shaped causal prefill: 8 prompts U[4096,32768], Hq=32 H=8 D=128",
                                   "bound": "mfma", "achieved": p["tflops_kernel"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": p["frac_of_mfma_peak"], "avg_launch_ms": p["kernel_ms"], "algorithmic_flops_per_launch": p["flops"],
                                   "traffic": (traffic or {}).get("total_bytes"), "traffic_measured_with": stamp, "traffic_detail": traffic}
        if "cpu_baseline" in p:
            prefill_cpu["C3"] = p["cpu_baseline"]
        pz = run_prefill(args, torch, W, wl3, iters=3, warmup=1, zero_operands=True)
        also["C3_llama3_8b_prefill"]["same_kernel_on_all_zero_operands"] = {
            "kernel_tflops": pz["tflops_kernel"], "frac_of_bf16_mfma_peak": pz["frac_of_mfma_peak"], "kernel_ms": pz["kernel_ms"],
            "note": "not a throughput claim: with zeros the chip holds its full clock, so this is the share of matrix-pipe cycles the "
                    "kernel fills; with N(0,1) operands the same instruction stream runs at the clock the power limit allows"}
    if args.only in ("all", "mixed"):
        wl4 = W.config(3)
        m4 = run_mixed(args, torch, W, wl4, max(20, args.steps // 5), 10)
        also["C4_yi34b_mixed_step"] = m4
        # the chunk alone (no other kernel between its launches), with the oracle on sampled rows
        p4 = run_prefill(args, torch, W, wl4, iters=9, warmup=2, oracle_rows=512 if oracle_on else 0,
                         name="the C4 chunk (2048 rows appended at 8192)")
        also["C4_yi34b_prefill_chunk_alone"] = {"kernel_tflops": p4["tflops_kernel"], "frac_of_bf16_mfma_peak": p4["frac_of_mfma_peak"],
                                                "kernel_ms": p4["kernel_ms"], "flops_per_launch": p4["flops"]}
        if "cpu_baseline" in p4:
            prefill_cpu["C4_chunk"] = p4["cpu_baseline"]
    if args.only in ("all", "c5"):
        wl5 = W.config(4)
        p5 = run_prefill(args, torch, W, wl5, iters=3, warmup=1, oracle_rows=512 if oracle_on else 0,
                         name="C5 (one 131072-token prompt)")
        also["C5_long_prefill_131072"] = {"kernel_tflops": p5["tflops_kernel"], "frac_of_bf16_mfma_peak": p5["frac_of_mfma_peak"],
                                          "kernel_ms": p5["kernel_ms"], "flops_per_launch": p5["flops"]}
        if "cpu_baseline" in p5:
            prefill_cpu["C5"] = p5["cpu_baseline"]
        wl5d = W.Workload("C5-decode", wl5.shape, wl5.seed, [1], [131072])
        d5 = run_decode(args, torch, W, wl5d, 256, 50, layers=2, with_oracle=False)
        also["C5_long_decode_131072"] = {"gbs_kernel": d5["gbs_kernel"], "frac_of_hbm_peak_kernel": d5["gbs_kernel"] / HBM_PEAK_GBS,
                                         "kernel_ms": d5["kernel_ms"], "ms_per_step": d5["ms_per_step"],
                                         "algorithmic_bytes_per_launch": d5["kbytes_per_launch"],
                                         "bytes_per_launch_over_all_launches": d5["bytes_per_launch_over_all_launches"]}
    if args.only in ("all", "prefill"):
        # Last, so that it does not warm the chip up before the measurements above: what a bf16 contraction can
        # reach at all here with N(0,1) data - a register-only MFMA loop on every CU.
        import paper_2405_04437_amd as P
        sus_t, sus_mhz = max(P.mfma_microbench(True, 100000) for _ in range(2))
        zero_t, zero_mhz = P.mfma_microbench(False, 100000)
        also["mfma_sustained"] = {"n01_operands_tflops": sus_t, "n01_operands_shader_mhz": sus_mhz,
                                  "zero_operands_tflops": zero_t, "zero_operands_shader_mhz": zero_mhz,
                                  "note": "register-only v_mfma_f32_32x32x16_bf16 loop on every CU; the chip lowers its clock "
                                          "for non-zero operands, so no bf16 contraction over N(0,1) data exceeds the first figure"}
        # the same loop with the side work of an attention inner loop added per matrix instruction, N(0,1) operands:
        # what each kind of work costs under the power limit
        side = {}
        for label, kw in (("mfma_only", {}), ("plus_lds_operand_read", {"lds_operand": True}), ("plus_3_fp32_fma", {"fma3": True}),
                          ("plus_1_exp2", {"exp2": True}), ("plus_all_three", {"lds_operand": True, "fma3": True, "exp2": True})):
            t, mhz = P.mfma_microbench(True, 60000, **kw)
            tz, mhzz = P.mfma_microbench(False, 60000, **kw)
            side[label] = {"n01_tflops": t, "n01_shader_mhz": mhz, "zero_operands_tflops": tz, "zero_operands_shader_mhz": mhzz}
        also["mfma_side_work_per_instruction"] = side
        for key in ("C3_llama3_8b_prefill", "C4_yi34b_prefill_chunk_alone", "C5_long_prefill_131072"):
            if key in also:
                also[key]["frac_of_sustained_n01_rate"] = also[key]["kernel_tflops"] / sus_t
        if "roofline_prefill" in out:
            out["roofline_prefill"]["sustained_n01_tflops"] = sus_t
            out["roofline_prefill"]["frac_of_sustained_n01_rate"] = out["roofline_prefill"]["achieved"] / sus_t
    if "roofline" in out and "roofline_prefill" in out:
        out["roofline"]["prefill"] = out["roofline_prefill"]     # the second half of the metric, inside the object the driver keeps
    if prefill_cpu:
        out.setdefault("cpu_baseline", {"kind": "oracle", "note": "decode leg not run"})["prefill"] = prefill_cpu
    if args.only == "prefill":
        p = also["C3_llama3_8b_prefill"]
        out["value"] = p["kernel_tflops"]; out["unit"] = "TFLOP/s"; out["ms_per_step"] = p["ms"]
        out["config"] = {"workload": out["roofline_prefill"]["workload"]}
        out["roofline"] = dict(out["roofline_prefill"])
    elif args.only == "mixed":
        m = also["C4_yi34b_mixed_step"]
        out["value"] = m["decode_gbs_kernel"]; out["ms_per_step"] = m["ms_per_step"]
        out["config"] = {"workload": "C4 Yi-34B-shaped mixed step: 128 decodes ctx U[2048,32768] + a 2048-token chunk at 8192, 10 % churn"}
    elif args.only == "c5":
        out["value"] = also["C5_long_decode_131072"]["gbs_kernel"]; out["ms_per_step"] = also["C5_long_decode_131072"]["ms_per_step"]
        out["config"] = {"workload": "C5 Llama-3-8B-shaped single request: 131072-token prefill, then 256 decode steps"}
    out["also"] = also
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
