"""Pins for the integer allocator model: figures the paper prints, Table 4 semantics, and
invariants (pool conservation, page-aligned sub-tensors, all-or-nothing step)."""
import os

import numpy as np
import pytest

import workloads as W
from oracle.allocator import AllocatorModel

GOLD = os.path.join(os.path.dirname(__file__), "golden")
KiB, MiB = 1024, 1024 * 1024
SHAPES = {"yi-6b": W.YI_6B, "llama-3-8b": W.LLAMA3_8B, "yi-34b": W.YI_34B}


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_tokens_per_page_group_table():
    for model, tp, heads, *tok in _rows("tokens_per_page_group.txt"):
        sh = SHAPES[model]
        assert sh.num_kv_heads // int(tp) == int(heads)
        for G, want in zip((64 * KiB, 128 * KiB, 256 * KiB, 2 * MiB), tok):
            m = AllocatorModel(sh.num_layers, 4, 200000, int(heads), sh.head_dim, 2, G, 0)
            assert m.tokens_per_page_group() == int(want)
            # a page-group is exhausted exactly after that many tokens
            assert m.need(int(want)) == 1 and m.need(int(want) + 1) == 2 and m.need(0) == 0


def test_per_token_footprint_all_layers():
    for model, layers, heads, kib in _rows("per_token_footprint.txt"):
        sh = SHAPES[model]
        assert (sh.num_layers, sh.num_kv_heads) == (int(layers), int(heads))
        m = AllocatorModel(sh.num_layers, 1, 1024, sh.num_kv_heads, sh.head_dim, 2, 64 * KiB, 0)
        assert 2 * m.N * m.token_bytes == int(kib) * KiB


def test_design_section_worked_example():
    vals = {k: int(v) for k, v in _rows("design_examples.txt")}
    m = AllocatorModel(60, 500, 200000, 4, 128, 2, 2 * MiB, 10 ** 6)
    assert m.token_bytes == 4 * 128 * 2
    assert abs(m.S - vals["yi34b_tp2_S_bytes_approx"]) / vals["yi34b_tp2_S_bytes_approx"] < 0.03
    assert m.S % m.G == 0 and m.S >= 200000 * 4 * 128 * 2
    assert abs(m.B * m.S - vals["yi34b_tp2_BS_bytes_approx"]) / vals["yi34b_tp2_BS_bytes_approx"] < 0.03
    assert abs(2 * m.N * m.B * m.S - vals["yi34b_total_va_bytes_approx"]) / vals["yi34b_total_va_bytes_approx"] < 0.03
    # growing one request by one page-group per sub-tensor = 120 mappings
    r = m.alloc_reqid()
    lens = [0] * 500
    lens[r] = 1
    assert m.step(lens) == 0
    assert m.map_calls == vals["yi34b_map_calls_per_request_page"]
    lens[r] = m.tokens_per_page_group() + 1
    assert m.step(lens) == 0
    assert m.map_calls == 2 * vals["yi34b_map_calls_per_request_page"]


def test_reqid_offsets_and_alignment():
    m = AllocatorModel(2, 7, 1000, 2, 64, 2, 64 * KiB, 100)
    assert m.S == 4 * 64 * KiB  # 1000*256 B = 250 KiB rounded up to 256 KiB
    for r in range(7):
        assert m.query(r)[2] == r * m.S and m.query(r)[2] % m.G == 0


def test_decode_maps_at_most_one_page_group_per_step():
    m = AllocatorModel(3, 2, 10000, 4, 128, 2, 64 * KiB, 10 ** 4)
    r = m.alloc_reqid()
    lens = [0, 0]
    prev = 0
    for n in range(1, 400):
        lens[r] = n
        assert m.step(lens) == 0
        now = m.query(r)[1]
        assert now - prev in (0, 1) and now == -(-n * m.token_bytes // m.G)
        prev = now
    assert sum(m.mapped) * 2 * m.N + m.pool_free == m.pool_total


def test_design_figure_walkthrough_deferred():
    """The five panels of the design figure: (a) two request slots, nothing mapped; (b) R1 gets one
    page; (c) R1 has two, R2 one; (d) R1 completes, its pages stay; (e) R3 arrives and is given
    R1's already backed tensor."""
    m = AllocatorModel(1, 2, 4096, 1, 128, 2, 64 * KiB, 8, policy="deferred")
    t = m.tokens_per_page_group()
    assert [m.query(r)[:2] for r in (0, 1)] == [(0, 0), (0, 0)]                     # (a)
    r1 = m.alloc_reqid()
    assert m.step([t if r == r1 else 0 for r in range(2)]) == 0
    assert m.query(r1)[:2] == (1, 1)                                                 # (b)
    r2 = m.alloc_reqid()
    lens = [0, 0]; lens[r1] = t + 1; lens[r2] = 5
    assert m.step(lens) == 0
    assert m.query(r1)[:2] == (1, 2) and m.query(r2)[:2] == (1, 1)                   # (c)
    assert m.free_reqid(r1) == 0
    assert m.query(r1)[:2] == (0, 2) and m.pool_free == 8 - 2 * 3                     # (d)
    r3 = m.alloc_reqid()
    assert r3 == r1 and m.query(r3)[:2] == (1, 2)                                    # (e)
    before = m.map_calls
    lens[r3] = 2 * t; assert m.step(lens) == 0
    assert m.map_calls == before  # no new mapping: the context fits what R1 left behind


def test_sync_policy_unmaps_on_free_and_reuses_lowest_id():
    m = AllocatorModel(2, 3, 4096, 2, 64, 2, 4 * KiB, 1000)
    a, b, c = m.alloc_reqid(), m.alloc_reqid(), m.alloc_reqid()
    assert (a, b, c) == (0, 1, 2) and m.alloc_reqid() == -1
    assert m.step([100, 200, 300]) == 0
    used = sum(m.mapped) * 4
    assert m.pool_free == 1000 - used
    assert m.free_reqid(b) == 0 and m.query(b)[:2] == (0, 0)
    assert m.free_reqid(b) == -1 and m.free_reqid(7) == -1
    assert m.alloc_reqid() == 1


def test_step_failure_changes_nothing():
    m = AllocatorModel(1, 2, 100000, 1, 128, 2, 64 * KiB, 6)
    a, b = m.alloc_reqid(), m.alloc_reqid()
    assert m.step([256, 256]) == 0  # 1 page-group each, K and V: 4 of 6 used
    snap = (list(m.mapped), m.pool_free)
    assert m.step([256, 1024]) == -1  # b would need 4 -> 6 more > 2 free
    assert (list(m.mapped), m.pool_free) == snap
    assert m.step([512, 256]) == 0 and m.pool_free == 0
    # invalid inputs
    assert m.step([1, 1, 1]) == -1
    assert m.step([100001, 1]) == -1
    m.free_reqid(b)
    assert m.step([512, 3]) == -1  # non-zero length for an inactive id


def test_deferred_reclaims_only_when_short_and_in_order():
    m = AllocatorModel(1, 3, 100000, 1, 128, 2, 64 * KiB, 12, policy="deferred")
    ids = [m.alloc_reqid() for _ in range(3)]
    assert ids == [0, 1, 2]
    assert m.step([512, 512, 512]) == 0 and m.pool_free == 0   # 2 page-groups x (K,V) x 3
    m.free_reqid(0); m.free_reqid(1)
    assert m.pool_free == 0 and m.mapped == [2, 2, 2]
    assert m.step([0, 0, 768]) == 0                            # needs 1 more row = 2 pages
    assert m.mapped == [1, 2, 3] and m.pool_free == 0          # taken from id 0, highest page
    assert m.step([0, 0, 2048]) == -1 and m.mapped == [1, 2, 3]  # needs 8 rows, only 3 reclaimable
    assert m.alloc_reqid() == 1                                # most pages mapped wins
    assert m.step([0, 1, 1536]) == -1 and m.mapped == [1, 2, 3]   # 3 more rows, 1 reclaimable
    assert m.step([0, 1, 1024]) == 0 and m.mapped == [0, 2, 4] and m.pool_free == 0


def test_conservation_on_a_random_trace():
    sh = W.TINY
    for policy in ("sync", "deferred"):
        m = AllocatorModel(sh.num_layers, 8, 2048, sh.num_kv_heads, sh.head_dim, 2, 16 * KiB, 400, policy)
        rng = np.random.default_rng(5)
        lens = [0] * 8
        for _ in range(500):
            x = rng.random()
            if x < 0.2:
                r = m.alloc_reqid()
                if r >= 0:
                    lens[r] = int(rng.integers(1, 600))
            elif x < 0.3:
                act = [r for r in range(8) if m.active[r]]
                if act:
                    r = int(rng.choice(act)); lens[r] = 0; assert m.free_reqid(r) == 0
            else:
                trial = [l + 1 if m.active[r] and l < 2048 else l for r, l in enumerate(lens)]
                if m.step(trial) == 0:
                    lens = trial
                    assert all(m.mapped[r] >= m.need(lens[r]) for r in range(8) if m.active[r])
            assert sum(m.mapped) * 2 * m.N + m.pool_free == m.pool_total
            assert m.pool_free >= 0


# ---- tensor slicing (Discussion section of the paper) ---------------------------------------------

def test_tokens_per_page_with_tensor_slicing_table():
    for model, tp, heads, without, with_, exact in _rows("tokens_per_page_sliced.txt"):
        sh = SHAPES[model]
        plain = AllocatorModel(sh.num_layers, 4, 4096, int(heads), sh.head_dim, 2, 2 * MiB, 0)
        sliced = AllocatorModel(sh.num_layers, 4, 4096, int(heads), sh.head_dim, 2, 2 * MiB, 0, sliced=True)
        assert plain.tokens_per_page_group() == int(without)
        quotient = 2 * MiB / (sh.num_layers * int(heads) * sh.head_dim * 2)
        if int(exact):
            assert sliced.tokens_per_page_group() == int(with_) == quotient
        else:  # printed: the TP-1 quotient rounded up (doubled for TP-2); whole tokens per page is the floor
            assert int(tp) * int(np.ceil(quotient / int(tp))) == int(with_)
            assert sliced.tokens_per_page_group() == int(np.floor(quotient))
        # fragmentation falls to 1/N of the unsliced design (up to the floor)
        assert plain.tokens_per_page_group() // sh.num_layers == sliced.tokens_per_page_group()
        t = sliced.tokens_per_page_group()
        assert sliced.need(t) == 1 and sliced.need(t + 1) == 2


def test_sliced_growth_takes_two_handles_per_page_group_and_same_bytes():
    N, H, D = 32, 8, 128
    plain = AllocatorModel(N, 2, 8192, H, D, 2, 2 * MiB, 10 ** 6)
    sliced = AllocatorModel(N, 2, 8192, H, D, 2, 2 * MiB, 10 ** 6, sliced=True)
    for m in (plain, sliced):
        r = m.alloc_reqid()
        assert m.step([8192, 0]) == 0
    # same physical bytes for a full-length request, N times fewer bytes for a one-token request
    assert plain.map_calls == sliced.map_calls == 2 * N * 8192 * H * D * 2 // (2 * MiB)
    assert sliced.S == N * plain.S and sliced.va_offset(1) == sliced.S
    a = AllocatorModel(N, 2, 8192, H, D, 2, 2 * MiB, 10 ** 6); a.alloc_reqid(); a.step([1, 0])
    b = AllocatorModel(N, 2, 8192, H, D, 2, 2 * MiB, 10 ** 6, sliced=True); b.alloc_reqid(); b.step([1, 0])
    assert a.map_calls == 2 * N and b.map_calls == 2


# ---- latency hiding (Sec. 6.1) ----------------------------------------------------------------------

def _decode_loop(m, lens, steps):
    for _ in range(steps):
        lens = [x + 1 if x else 0 for x in lens]
        assert m.step(lens) == 0
    return lens


def test_lookahead_takes_decode_growth_off_the_critical_path():
    kw = dict(N=2, B=4, L=5000, H=4, D=128, P=2, page_group_bytes=64 * KiB, pool_page_groups=4000)
    sync = AllocatorModel(**kw)
    over = AllocatorModel(**kw, background=True, lookahead_tokens=1)
    lens = [100, 37, 0, 0]
    for m in (sync, over):
        m.alloc_reqid(); m.alloc_reqid()
        assert m.step(lens) == 0
    first = over.sync_map_calls
    _decode_loop(sync, lens, 300); _decode_loop(over, lens, 300)
    # every page-group a decode step needs was mapped by the pass after the previous step
    assert over.sync_map_calls == first and over.background_map_calls > 0
    # the overlapped manager is never behind and at most one token's worth of page-groups ahead
    for r in range(4):
        assert sync.mapped[r] <= over.mapped[r] <= sync.mapped[r] + 1
    assert over.sync_map_calls + over.background_map_calls == over.map_calls
    assert sync.sync_map_calls == sync.map_calls and sync.background_map_calls == 0


def test_lookahead_skips_what_does_not_fit_and_never_fails_step():
    m = AllocatorModel(1, 2, 1000, 1, 64, 2, 4 * KiB, pool_page_groups=4, background=True, lookahead_tokens=32)
    a, b = m.alloc_reqid(), m.alloc_reqid()
    assert m.step([32, 32]) == 0          # 2 rows * 2 buffers = 4 page-groups: pool empty, nothing to look ahead with
    assert m.mapped == [1, 1] and m.pool_free == 0
    assert m.step([33, 32]) == -1         # the demand itself still fails as before
    assert m.mapped == [1, 1]


def test_eager_allocation_backs_the_next_reqid():
    m = AllocatorModel(2, 4, 4096, 2, 64, 2, 4 * KiB, pool_page_groups=400, policy="deferred", background=True,
                       eager_page_groups=3)
    r0 = m.alloc_reqid()
    assert m.step([10, 0, 0, 0]) == 0
    cand = m.next_candidate()
    assert cand == 1 and m.mapped[cand] == 3            # topped up by the background pass
    sync_before = m.sync_map_calls
    r1 = m.alloc_reqid()
    assert r1 == cand
    lens = [10, 3 * m.tokens_per_page_group(), 0, 0]
    assert m.step(lens) == 0
    assert m.sync_map_calls == sync_before              # the prefill found its pages mapped
    assert m.mapped[m.next_candidate()] == 3            # and a new candidate was prepared
    # a finished request keeps its pages and becomes the preferred candidate when it holds more
    assert m.free_reqid(r1) == 0 and m.next_candidate() in (r1, 2)
    assert m.pool_free + m.nbuf * sum(m.mapped) == m.pool_total


def test_threshold_reclaim_spares_the_candidate_and_stops_at_the_threshold():
    m = AllocatorModel(1, 4, 4096, 1, 64, 2, 4 * KiB, pool_page_groups=40, policy="deferred", background=True,
                       reclaim_threshold=10)
    ids = [m.alloc_reqid() for _ in range(4)]
    t = m.tokens_per_page_group()
    assert m.step([5 * t, 4 * t, 4 * t, 4 * t]) == 0     # 17 rows * 2 = 34 page-groups, 6 free
    assert m.pool_free == 6
    for r in (0, 1, 2):
        m.free_reqid(r)
    assert m.mapped == [5, 4, 4, 4]                      # deferred: nothing unmapped yet
    assert m.step([0, 0, 0, 4 * t]) == 0
    # candidate = id 0 (most pages) is spared; id 1 gives back from the top until 10 are free
    assert m.mapped == [5, 2, 4, 4] and m.pool_free == 10
    assert m.unmap_calls == 4


def test_background_conservation_on_a_random_trace():
    rng = np.random.default_rng(77)
    m = AllocatorModel(3, 8, 3000, 2, 64, 2, 8 * KiB, pool_page_groups=900, policy="deferred", background=True,
                       lookahead_tokens=1, eager_page_groups=2, reclaim_threshold=120)
    lens = [0] * 8
    for _ in range(600):
        op = rng.integers(0, 10)
        if op == 0:
            r = m.alloc_reqid()
            if r >= 0:
                lens[r] = int(rng.integers(1, 1500))
        elif op == 1:
            act = [r for r in range(8) if m.active[r]]
            if act:
                r = int(rng.choice(act)); m.free_reqid(r); lens[r] = 0
        else:
            trial = [min(x + 1, 3000) if x else 0 for x in lens]
            if m.step(trial) == 0:
                lens = trial
                for r in range(8):
                    if m.active[r]:
                        assert m.mapped[r] >= m.need(lens[r])
        assert m.pool_free >= 0 and m.pool_free + m.nbuf * sum(m.mapped) == m.pool_total
