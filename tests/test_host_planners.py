"""The launch planners built for the host.  Decode split-K planner (csrc/decode_plan.h): whatever the batch, the segments it
describes - recomputed here the way the kernels do, from `period` and the nine prefix values - cover every
tile exactly once in order, stay inside the workspace bound, follow the per-XCD weights, and give every
(segment, request) pair its own partial slot.  Prefill work queues (csrc/prefill_plan.h): every (request, KV head,
query tile) sits in exactly one of the eight queues, longest first, padding only at the tails."""
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
BUILD = os.path.join(HERE, "host", "_build")


@pytest.fixture(scope="module")
def planner():
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "plan_harness")
    r = subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", os.path.join(HERE, "host", "plan_harness.cpp"), "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    p = subprocess.Popen([exe], stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)

    def ask(chunk, resident, per_slot, weights, lens):
        p.stdin.write(" ".join(str(x) for x in [chunk, resident, per_slot, *weights, *lens]) + "\n")
        p.stdin.flush()
        v = [int(x) for x in p.stdout.readline().split()]
        return {"total": v[0], "num_segs": v[1], "max_segs": v[2], "period": v[3], "pre": v[4:13]}

    def queues(Hq, H, cus, q_lens, kv_lens):
        flat = [v for pair in zip(q_lens, kv_lens) for v in pair]
        p.stdin.write(" ".join(str(x) for x in ["Q", Hq, H, cus, len(q_lens), *flat]) + "\n")
        p.stdin.flush()
        v = [int(x) for x in p.stdout.readline().split()]
        items = np.array(v[3:], dtype=np.int64).reshape(8, v[2], 7) if v[2] else np.zeros((8, 0, 7), dtype=np.int64)
        return {"waves": v[0], "rows": v[1], "per_xcd": v[2], "items": items}

    ask.queues = queues
    yield ask
    p.stdin.close()
    p.wait(timeout=30)


def seg_range(plan, s):
    """What decode_splitk_kernel computes for workgroup s."""
    t0 = min((s >> 3) * plan["period"] + plan["pre"][s & 7], plan["total"])
    t1 = min((s >> 3) * plan["period"] + plan["pre"][(s & 7) + 1], plan["total"])
    return t0, t1


def seg_of(plan, t):
    """What the reduce kernels compute for tile t."""
    p, r = divmod(t, plan["period"])
    return p * 8 + sum(1 for i in range(1, 8) if r >= plan["pre"][i])


def check_plan(plan, lens, grid_pad=16):
    tiles = [(L + 31) // 32 for L in lens]
    assert plan["total"] == sum(tiles)
    assert plan["pre"][0] == 0 and plan["pre"][8] == plan["period"] > 0
    assert all(a <= b for a, b in zip(plan["pre"], plan["pre"][1:]))
    # the segments up to num_segs tile the sequence in order; the padding workgroups of a launch get nothing
    at = 0
    for s in range(plan["num_segs"]):
        t0, t1 = seg_range(plan, s)
        assert t0 == at and t1 > t0          # no empty segment inside the sequence: the reduce kernels read every slot
        at = t1
    assert at == plan["total"]
    for s in range(plan["num_segs"], plan["num_segs"] + grid_pad):
        t0, t1 = seg_range(plan, s)
        assert t0 == t1
    # every tile's segment, found the reduce kernel's way, is the one whose range holds it (sampled)
    rng = np.random.default_rng(plan["total"])
    for t in set([0, plan["total"] - 1] + rng.integers(0, plan["total"], size=64).tolist()):
        s = seg_of(plan, t)
        t0, t1 = seg_range(plan, s)
        assert t0 <= t < t1 and s < plan["num_segs"]
    # partial slots: (segment of a request's tile) + request index never repeats along the sequence
    cu = np.concatenate([[0], np.cumsum(tiles)])
    last = -1
    for r in range(len(lens)):
        c0, c1 = seg_of(plan, int(cu[r])) + r, seg_of(plan, int(cu[r + 1]) - 1) + r
        assert c0 > last and c1 >= c0 and c1 < plan["num_segs"] + len(lens)
        last = c1


DEFAULT_W = [1, 0.9] * 4


@pytest.mark.parametrize("resident,per_slot", [(256, 1), (128, 1), (256, 4), (304, 1), (4, 1)])
def test_default_mode_covers_every_tile_once_and_fits_the_bound(planner, resident, per_slot):
    rng = np.random.default_rng(resident * 7 + per_slot)
    cases = [[1], [32], [33], [131072], [1] * 300, rng.integers(1, 512, size=4).tolist(),
             rng.integers(1024, 16384, endpoint=True, size=64).tolist(), rng.integers(2048, 32768, endpoint=True, size=128).tolist(),
             rng.integers(1, 100000, size=17).tolist()]
    for lens in cases:
        plan = planner(0, resident, per_slot, DEFAULT_W, lens)
        check_plan(plan, lens)
        assert plan["num_segs"] <= plan["max_segs"]


@pytest.mark.parametrize("chunk", [32, 64, 512, 4096])
def test_chunk_mode_cuts_equal_segments(planner, chunk):
    lens = [5000, 1, 777, 4096, 31, 20000]
    plan = planner(chunk, 256, 1, DEFAULT_W, lens)
    check_plan(plan, lens)
    assert plan["period"] == 8 * chunk // 32 and plan["pre"] == [x * chunk // 32 for x in range(9)]
    assert plan["num_segs"] == -(-plan["total"] // (chunk // 32))


@pytest.mark.parametrize("weights", [[1] * 8, DEFAULT_W, [4, 0.25, 1, 1, 0.25, 4, 2, 0.5], [0.25] * 7 + [4]])
def test_segment_lengths_follow_the_weights(planner, weights):
    lens = np.random.default_rng(5).integers(1024, 16384, endpoint=True, size=64).tolist()
    plan = planner(0, 256, 1, weights, lens)
    check_plan(plan, lens)
    lengths = np.diff(plan["pre"])
    want = plan["period"] * np.array(weights) / sum(weights)
    assert np.all(np.abs(lengths - want) < 1.0)          # largest-remainder rounding: off by less than one tile
    assert plan["num_segs"] <= 256 and plan["num_segs"] > 256 - 8    # one round of the resident workgroups


def test_a_weight_that_rounds_to_zero_tiles_still_gets_a_tile(planner):
    """One long request, weights at the ends of the accepted range: 0.25 / 28.25 of a 70-tile period is less than a
    tile.  Every partial slot the reduce kernel reads for the request must belong to a non-empty segment."""
    weights = [0.25] + [4] * 7
    lens = [71680]                                     # 2240 tiles over 32 periods: 70 tiles per period
    plan = planner(0, 256, 1, weights, lens)
    check_plan(plan, lens)
    assert min(np.diff(plan["pre"])) >= 1 and plan["period"] == 70
    first, last = seg_of(plan, 0), seg_of(plan, plan["total"] - 1)
    for s in range(first, last + 1):
        t0, t1 = seg_range(plan, s)
        assert t1 > t0


def test_short_batches_fall_back_to_equal_segments(planner):
    plan = planner(0, 256, 1, [4, 0.25, 1, 1, 0.25, 4, 2, 0.5], [100, 200, 50])       # 13 tiles
    check_plan(plan, [100, 200, 50])
    assert len(set(np.diff(plan["pre"]).tolist())) == 1 and plan["num_segs"] == 13


@pytest.mark.parametrize("Hq,H", [(32, 8), (56, 8), (32, 4), (8, 2), (3, 3), (7, 1), (64, 16)])
def test_prefill_queues_hold_every_work_item_once(planner, Hq, H):
    rng = np.random.default_rng(Hq * 31 + H)
    cases = [([0], [5]), ([1], [1]), ([300, 200, 1, 77, 0, 513], [1300, 200, 555, 400, 10, 577]),
             (rng.integers(4096, 32768, endpoint=True, size=8).tolist(),) * 2, ([2048], [10240]), ([131072], [131072])]
    for q_lens, kv_lens in cases:
        pq = planner.queues(Hq, H, 256, q_lens, kv_lens)
        many = sum(-(-q // 384) for q in q_lens) * Hq >= 4 * 256
        assert pq["waves"] == (12 if many else 8)
        BM = pq["rows"]
        assert BM == 32 * pq["waves"]
        want = {(r, kvh, t) for r, q in enumerate(q_lens) for t in range(-(-q // BM)) for kvh in range(H)}
        seen = []
        for x in range(8):
            queue = pq["items"][x]
            live = queue[queue[:, 0] >= 0]
            assert np.all(queue[len(live):, 0] == -1)                     # padding only at the tail
            seen += [tuple(int(v) for v in it[:3]) for it in live]
            cu = np.concatenate([[0], np.cumsum(q_lens)])
            for r, _, _, reqid, q_begin, q_len, kv_len in live:              # the record carries the request's own figures
                assert (reqid, q_begin, q_len, kv_len) == (1000 + 7 * r, cu[r], q_lens[r], kv_lens[r])
            cost = [min((t + 1) * BM, q_lens[r]) + kv_lens[r] - q_lens[r] for r, _, t in live[:, :3]]
            assert all(a >= b for a, b in zip(cost, cost[1:]))            # longest first
        assert len(seen) == len(want) and set(seen) == want
        assert pq["per_xcd"] * 8 >= len(want) and (pq["per_xcd"] == 0) == (len(want) == 0)


def test_prefill_queues_keep_a_kv_stream_on_one_xcd(planner):
    """All query tiles of one (request, KV head) - or of one tile class when there are fewer than 8 KV heads - share a queue."""
    pq = planner.queues(32, 8, 256, [5000, 9000, 4097], [5000, 9000, 5097])
    home = {}
    for x in range(8):
        for r, kvh, t in pq["items"][x][:, :3]:
            if r >= 0:
                assert home.setdefault((int(r), int(kvh)), x) == x
    pq = planner.queues(32, 4, 256, [5000, 9000, 4097], [5000, 9000, 5097])       # 4 KV heads: two tile classes each
    home = {}
    for x in range(8):
        for r, kvh, t in pq["items"][x][:, :3]:
            if r >= 0:
                assert home.setdefault((int(r), int(kvh), int(t) % 2), x) == x
