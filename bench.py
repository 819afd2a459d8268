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
launch on the launch stream.  `also.C2_one_layer_per_sync` is the same batch with a host synchronisation
after each single layer, which exposes the per-iteration host work instead of amortising it.

The line also carries `also`: prefill (config 3) TFLOP/s, the mixed step of config 4 and the
long-context request of config 5, each with its own roofline fraction, and `cpu_baseline`: the CPU
oracle timed on the same decode batch.

Synthetic data: N(0,1) bf16 Q/K/V drawn on the device from a seeded generator; context lengths from
workloads.config().  Nothing is read from disk except the optional measured-traffic file under
profiles/ (rocprofv3 counter results for the same command).
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


def _prefill_flops(shape, q_lens, kv_lens):
    """Causal-only flops: 4*Hq*D per (query row, visible key) pair."""
    tot = 0
    for ql, kl in zip(q_lens, kv_lens):
        off = kl - ql
        tot += ql * off + ql * (ql + 1) // 2
    return 4 * shape.num_q_heads * shape.head_dim * tot


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
            k = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            v = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            for layer in range(layers):
                sess.append(layer, k, v, [r], [0, n], [done])
            if keep_host:
                ks.append(k.cpu()); vs.append(v.cpu())
            done += n
        if keep_host:
            host.append((torch.cat(ks), torch.cat(vs)))
    torch.cuda.synchronize()
    return ids, host


def run_decode(args, torch, W, wl, steps, warmup, layers=2, with_oracle=True, churn=False, whole_model=False,
               background=False):
    """Decode steps.  whole_model=False: one layer's attention per step (the layer rotates) and a stream
    synchronisation after it.  whole_model=True: a serving iteration - step() once, then the fused
    append + attention of every one of `layers` layers, then the synchronisation (Algorithm 1)."""
    from paper_2405_04437_amd import FLAG_BACKGROUND, POLICY_DEFERRED
    from paper_2405_04437_amd.runtime import KvSession, tensor_to_bits, tensor_to_f32

    shape = wl.shape
    n = sum(1 for q in wl.q_lens if q == 1)
    kv_lens = [int(x) for x in wl.kv_lens[:n]]
    ksteps = max(1, steps // 8) if whole_model else steps     # steps of the second, event-timed pass
    total_steps = steps + ksteps + warmup + 2
    ctx_hi = wl.extra["ctx_range"][1] if churn else 0
    max_ctx = max(max(kv_lens), ctx_hi) + total_steps + 8 + 64
    G = 2 * MiB
    headroom = n // 4 + 4
    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    budget = per_req * 2 * layers * (n + headroom)
    lookahead = 64 if background else 0
    if not churn:   # the page-groups these requests can reach by the last step (look-ahead included), and a few spare rows
        rows = sum((int(L + total_steps + 8 + lookahead) * shape.token_bytes + G - 1) // G for L in kv_lens) + 8
        budget = rows * G * 2 * layers
    sess = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n + headroom, max_ctx, budget, layers, G,
                     POLICY_DEFERRED, flags=FLAG_BACKGROUND if background else 0,
                     lookahead_tokens=lookahead)
    gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    ids, host = _fill_contexts(sess, torch, gen, shape, kv_lens, layers, keep_host=with_oracle)
    for r, L in zip(ids, kv_lens):
        sess.seq_lens[r] = L
    scale = W.softmax_scale(shape.head_dim)
    q = torch.randn((n, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    knew = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    vnew = torch.randn((n, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    o = torch.empty_like(q)
    import numpy as np
    lens = np.array(kv_lens, dtype=np.int64)
    ids = np.array(ids, dtype=np.int32)
    seq = np.zeros(sess.B, dtype=np.int64)      # cache_seq_len of Algorithm 1, indexed by reqId
    ws = sess.workspace([max(int(L), ctx_hi) + total_steps for L in lens])
    if churn:  # source rows for the K/V of newly arriving requests (their prefill's KV write)
        kbig = torch.randn((ctx_hi, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        vbig = torch.randn((ctx_hi, shape.num_kv_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    cu = np.arange(n + 1, dtype=np.int32)
    rng = np.random.default_rng(wl.seed)
    per_tok = 2 * shape.num_kv_heads * shape.head_dim * 2
    qo_bytes = n * 2 * shape.num_q_heads * shape.head_dim * 2
    va, stream = sess.va, sess.stream
    torch_stream = torch.cuda.current_stream()

    def one_step(i):
        arrivals = []
        if churn:  # config 4: ~10% of the requests finish and as many arrive, reusing backed reqIds
            k = max(1, int(round(0.10 * n)))
            for slot in rng.choice(n, size=k, replace=False):
                seq[ids[slot]] = 0
                assert va.free_reqid(int(ids[slot])) == 0
                lens[slot] = int(rng.integers(wl.extra["ctx_range"][0], wl.extra["ctx_range"][1], endpoint=True))
                ids[slot] = va.alloc_reqid()
                arrivals.append(slot)
        seq[ids] = lens + 1                # newcomers: their context and its first generated token
        assert va.step(seq) == 0
        if churn:
            # The memory management above ran while the GPU was still busy with the previous iteration (Sec. 6.1.1
            # of the paper: allocation overlapped with compute; nothing is unmapped under the deferred policy, and
            # mapping does not disturb running kernels).  That iteration's output is needed before this one is launched.
            torch_stream.synchronize()
            for slot in arrivals:  # the newcomer's context is written in place (contiguous copy)
                L = int(lens[slot])
                for layer in range(layers):
                    assert va.append_kv(layer, stream, kbig[:L], vbig[:L], ids[slot:slot + 1], [0, L], [0]) == 0
        if whole_model:                   # every layer: the new K/V row rides in that layer's decode kernel
            for layer in range(layers):
                assert va.attn_decode_append(layer, stream, q, knew, vnew, o, ids, lens + 1, scale, ws, ws.numel()) == 0
        else:
            att = i % layers              # the layer attended to in this step; its append rides in the decode kernel
            assert va.attn_decode_append(att, stream, q, knew, vnew, o, ids, lens + 1, scale, ws, ws.numel()) == 0
            for layer in range(layers):   # the other layers' appends are independent of it and queue up behind
                if layer != att:
                    assert va.append_kv(layer, stream, knew, vnew, ids, cu, lens) == 0
        lens[:] += 1
        if not churn:
            # iteration boundary of the serving loop (Algorithm 1): the framework needs this iteration's
            # output on the host before it can schedule the next one
            torch_stream.synchronize()

    launches_per_step = layers if whole_model else 1

    def step_bytes():
        return (int(lens.sum()) * per_tok + qo_bytes) * launches_per_step

    for i in range(warmup):
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
    sess.va.kernel_time(0); sess.va.kernel_time(2)
    kbytes = 0
    for i in range(ksteps):
        one_step(warmup + steps + i)
        kbytes += step_bytes()
    torch.cuda.synchronize()
    k_ms, k_n = sess.va.kernel_time(0)
    r_ms, r_n = sess.va.kernel_time(2)
    sess.va.set_timing(False)
    kbytes_per_launch = kbytes / max(k_n, 1)
    ms_per_step = (t1 - t0) * 1e3 / steps
    bytes_per_step = bytes_total / steps
    res = {
        "ms_per_step": ms_per_step,
        "gbs_step": bytes_per_step / (ms_per_step * 1e6),
        "kernel_ms": k_ms / max(k_n, 1),
        "reduce_ms": r_ms / max(r_n, 1),
        "gbs_kernel": kbytes_per_launch / (k_ms / max(k_n, 1) * 1e6),
        "bytes_per_step": bytes_per_step,
        "kbytes_per_launch": kbytes_per_launch,
        "tokens_in_batch": int(lens.sum()),
        "layers": layers, "decode_launches_per_step": launches_per_step,
        "map_calls_in_timed_region": map1[0] - map0[0],
        "map_us_in_timed_region": map1[2] - map0[2],
        "unmap_calls_in_timed_region": map1[1] - map0[1],
    }
    if with_oracle and not churn:
        # CPU oracle on the same batch as the last timed step (layer = last used layer).
        import numpy as np
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
        reps = 4   # ~20 core-seconds of oracle work on a 16-core host
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


def run_prefill(args, torch, W, wl, iters, warmup, req_filter=None):
    from paper_2405_04437_amd.runtime import KvSession

    shape = wl.shape
    idx = [i for i, ql in enumerate(wl.q_lens) if ql > 1] if req_filter is None else req_filter
    q_lens = [int(wl.q_lens[i]) for i in idx]
    kv_lens = [int(wl.kv_lens[i]) for i in idx]
    n = len(idx)
    G = 2 * MiB
    max_ctx = max(kv_lens)
    per_req = (max_ctx * shape.token_bytes + G - 1) // G * G
    sess = KvSession(shape.num_q_heads, shape.num_kv_heads, shape.head_dim, n, max_ctx, per_req * 2 * n, 1, G)
    gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    ids, _ = _fill_contexts(sess, torch, gen, shape, kv_lens, 1)
    cu = [0]
    for ql in q_lens:
        cu.append(cu[-1] + ql)
    q = torch.empty((cu[-1], shape.num_q_heads, shape.head_dim), device="cuda", dtype=torch.bfloat16)
    for a in range(0, cu[-1], 16384):
        b = min(cu[-1], a + 16384)
        q[a:b] = torch.randn((b - a, shape.num_q_heads, shape.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
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
    sess.close()
    return {"ms_per_call": ms, "kernel_ms": kms, "tflops_call": flops / (ms * 1e9), "tflops_kernel": flops / (kms * 1e9),
            "frac_of_mfma_peak": flops / (kms * 1e9) / MFMA_BF16_PEAK_TFLOPS, "flops": flops, "q_tokens": cu[-1],
            "kernel_ms_per_launch": [round(x, 4) for x in per_launch]}


def _measured_traffic(name):
    p = os.path.join(ROOT, "profiles", "measured_traffic.json")
    try:
        with open(p) as f:
            return json.load(f).get(name)
    except Exception:
        return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps; the first ~50 ms of sustained load on a fresh process contain a one-off "
                         "30-40 ms device stall (seen between two back-to-back launches), so keep this >= 10 "
                         "whole-model steps")
    ap.add_argument("--only", choices=["all", "decode", "prefill", "copy"], default="all")
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
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "C2 Yi-6B-shaped decode: 64 requests, Hq=32 H=4 D=128, ctx U[1024,16384], "
                                  "one token per request per step (step() + per layer: K/V append fused into split-K decode, + reduce), 2 MiB page-groups"}}
    also = {}
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
        r = run_decode(args, torch, W, wl, args.steps, args.warmup, layers=depth, with_oracle=not args.no_cpu_baseline,
                       whole_model=True, background=not args.sync_maps)
        out["config"].update({"layers": depth, "decode_launches_per_step": depth,
                              "kv_growth": "step() on the caller's thread" if args.sync_maps else "helper thread, 64-token look-ahead"})
        out["value"] = r["gbs_step"]
        out["ms_per_step"] = r["ms_per_step"]
        out["pct_of_hbm_peak"] = 100.0 * r["gbs_step"] / HBM_PEAK_GBS
        out["roofline"] = {"kernel": "decode_splitk_kernel<128>", "bound": "hbm", "achieved": r["gbs_kernel"],
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": r["gbs_kernel"] / HBM_PEAK_GBS,
                           "avg_launch_ms": r["kernel_ms"], "algorithmic_bytes_per_launch": r["kbytes_per_launch"],
                           "traffic": (_measured_traffic("decode_splitk_C2") or {}).get("total_bytes"),
                           "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                           "traffic_detail": _measured_traffic("decode_splitk_C2")}
        if "cpu_baseline" in r:
            out["cpu_baseline"] = r.pop("cpu_baseline")
        out["decode_detail"] = {k: r[k] for k in ("reduce_ms", "tokens_in_batch", "map_calls_in_timed_region",
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
    if args.only in ("all", "prefill"):
        wl3 = W.config(2)
        p = run_prefill(args, torch, W, wl3, iters=7, warmup=2)
        also["C3_llama3_8b_prefill"] = {"tflops": p["tflops_call"], "kernel_tflops": p["tflops_kernel"],
                                        "frac_of_bf16_mfma_peak": p["frac_of_mfma_peak"],
                                        "ms": p["ms_per_call"],
                                        "kernel_ms": p["kernel_ms"], "kernel_ms_per_launch": p["kernel_ms_per_launch"], "q_tokens": p["q_tokens"],
                                        "flop_convention": "causal only: 4*Hq*D per visible (query,key) pair",
                                        "traffic": (_measured_traffic("prefill_C3") or {}).get("total_bytes"),
                                        "traffic_detail": _measured_traffic("prefill_C3")}
    if args.only == "all":
        wl4 = W.config(3)
        d4 = run_decode(args, torch, W, wl4, max(20, args.steps // 5), 10, layers=1, with_oracle=False, churn=True)
        also["C4_yi34b_mixed_decode_part"] = {"gbs_step": d4["gbs_step"], "gbs_kernel": d4["gbs_kernel"],
                                              "frac_of_hbm_peak_kernel": d4["gbs_kernel"] / HBM_PEAK_GBS,
                                              "ms_per_step": d4["ms_per_step"], "kernel_ms": d4["kernel_ms"],
                                              "map_calls": d4["map_calls_in_timed_region"], "map_us": d4["map_us_in_timed_region"],
                                              "unmap_calls": d4["unmap_calls_in_timed_region"]}
        p4 = run_prefill(args, torch, W, wl4, iters=9, warmup=2)
        also["C4_yi34b_prefill_chunk"] = {"kernel_tflops": p4["tflops_kernel"], "frac_of_bf16_mfma_peak": p4["frac_of_mfma_peak"],
                                          "kernel_ms": p4["kernel_ms"]}
        wl5 = W.config(4)
        p5 = run_prefill(args, torch, W, wl5, iters=3, warmup=1)
        also["C5_long_prefill_131072"] = {"kernel_tflops": p5["tflops_kernel"], "frac_of_bf16_mfma_peak": p5["frac_of_mfma_peak"],
                                          "kernel_ms": p5["kernel_ms"]}
        wl5d = W.Workload("C5-decode", wl5.shape, wl5.seed, [1], [131072])
        d5 = run_decode(args, torch, W, wl5d, 256, 50, layers=2, with_oracle=False)
        also["C5_long_decode_131072"] = {"gbs_kernel": d5["gbs_kernel"], "frac_of_hbm_peak_kernel": d5["gbs_kernel"] / HBM_PEAK_GBS,
                                         "kernel_ms": d5["kernel_ms"], "ms_per_step": d5["ms_per_step"]}
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
        for key in ("C3_llama3_8b_prefill", "C4_yi34b_prefill_chunk", "C5_long_prefill_131072"):
            if key in also:
                also[key]["frac_of_sustained_n01_rate"] = also[key]["kernel_tflops"] / sus_t
    if args.only == "prefill":
        p = also["C3_llama3_8b_prefill"]
        out["value"] = p["kernel_tflops"]; out["unit"] = "TFLOP/s"; out["ms_per_step"] = p["ms"]
        out["config"] = {"workload": "C3 Llama-3-8B-shaped causal prefill: 8 prompts U[4096,32768], Hq=32 H=8 D=128"}
        out["roofline"] = {"kernel": "prefill_kernel<128>", "bound": "mfma", "achieved": p["kernel_tflops"],
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": p["frac_of_bf16_mfma_peak"],
                           "traffic": p["traffic"]}
    out["also"] = also
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
