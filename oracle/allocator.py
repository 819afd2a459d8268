"""Integer model of the KV-cache memory manager (reserve / map / grow / free bookkeeping).

TEST INFRASTRUCTURE ONLY: nothing on the product path imports this module, and it shares no code
with the C++ allocator.  It follows the paper's design section:

* Sec. 5.1.2: 2*N virtual buffers per worker (K and V for each of the N layers).
* Sec. 5.1.3: each buffer has size B*S with S = L*H*D*P, the largest per-layer K (or V) cache of one
  request.  Here S is additionally rounded up to the page-group size so that every request's
  sub-tensor starts on a page boundary (Sec. 5.2.1 requires buffer and handle sizes to be multiples
  of the allocation granularity; applying that to S as well is this model's reading).
* Sec. 5.2.3: a request's sub-tensor sits at byte offset reqId * S in every buffer; reqId in [0,B).
* Table 4: init / alloc_reqid / free_reqid / step and their return values.
* Sec. 5.3.3: if one layer's K cache of a request needs s bytes and the page-group size is t, at
  least (s + t - 1) / t page-groups must be mapped in each of the 2*N sub-tensors; on unmet demand
  step() fails (-1).
* Sec. 5.3.4 / 6.1.2: a freed reqId's pages are either unmapped at once (policy "sync") or left
  mapped and handed, together with the reqId, to the next request (policy "deferred").

Readings where the paper is silent (kept deterministic so the library can match bit-exactly):
* alloc_reqid returns the lowest unused id under "sync"; under "deferred" the unused id with the
  most mapped page-groups, ties to the lowest id.
* step() is all-or-nothing: it first totals the demand of all active requests; if the free pool
  (plus, under "deferred", what inactive ids still hold) cannot cover it, nothing changes.
* A non-zero length for an inactive id, a length above L, or a wrong array size fails (-1).
  Lengths that shrink never unmap while the id is active.
* Under "deferred", step() reclaims only when the free pool is short: inactive ids in ascending
  order, each from its highest mapped page-group downwards, until the demand fits.
* The pool counts physical page-groups; growing one request by one page-group takes 2*N of them
  (the same page index in every buffer), so K and V counts are always equal.

Extensions beyond the base design (each switched on by a constructor argument):

* Tensor slicing (Sec. 8.2): one K and one V buffer of shape [B, L, N, H, D] instead of 2*N buffers,
  so a page-group holds the tokens of all layers: a token then takes N*H*D*P bytes of a buffer and
  growing a request by one page-group takes 2 handles.  The paper's table prints whole tokens per
  2 MiB page; the model uses the floor (Yi-34B: 2 MiB / (60*2048 B) = 17.07 -> 17, printed as 18).
* Latency hiding (Sec. 6.1): after a successful step() a background pass runs.  The library runs it
  on a thread and joins it before the next call that looks at the state, so the state seen at every
  call boundary is the one computed here in program order:
    1. look-ahead (Sec. 6.1.1): every active request with a non-zero length gets the page-groups
       that `lookahead_tokens` more tokens would need (capped at L), in ascending reqId order,
       from the free pool only; a request whose growth does not fit is skipped;
    2. threshold reclamation (Sec. 6.1.2, "deferred" only): if fewer than `reclaim_threshold`
       page-groups are free, inactive ids other than the next allocation candidate give pages
       back, ascending id, highest page-group first, until the threshold is met;
    3. eager allocation (Sec. 6.1.2, "deferred" only): the inactive id alloc_reqid would return
       next is topped up to `eager_page_groups`, as far as whole rows fit the free pool.
  The paper leaves the amounts open (it names no count and gives 10 % only as an example): they are parameters.

Parity status: pinned against the figures the paper prints (tokens per page-group table, per-token
footprints, the 120-calls-per-request-page example, the five-panel walk-through of the design
figure) in tests/test_oracle_allocator.py.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


class AllocatorModel:
    def __init__(self, N: int, B: int, L: int, H: int, D: int, P: int, page_group_bytes: int,
                 pool_page_groups: int, policy: str = "sync", sliced: bool = False, background: bool = False,
                 lookahead_tokens: int = 0, eager_page_groups: int = 0, reclaim_threshold: int = 0) -> None:
        if min(N, B, L, H, D, P, page_group_bytes) <= 0 or pool_page_groups < 0:
            raise ValueError("non-positive parameter")
        if policy not in ("sync", "deferred"):
            raise ValueError(policy)
        self.N, self.B, self.L, self.H, self.D, self.P = N, B, L, H, D, P
        self.G = page_group_bytes
        self.policy = policy
        self.sliced = sliced
        self.nbuf = 2 if sliced else 2 * N                # virtual buffers (handles per page-group row)
        self.token_bytes = (N if sliced else 1) * H * D * P   # one token in one buffer
        self.background = background
        self.lookahead_tokens, self.eager_page_groups, self.reclaim_threshold = lookahead_tokens, eager_page_groups, reclaim_threshold
        if min(lookahead_tokens, eager_page_groups, reclaim_threshold) < 0:
            raise ValueError("negative background parameter")
        self.sync_map_calls = 0                           # mappings done inside step() itself
        self.background_map_calls = 0                     # mappings done by the background pass
        raw = L * self.token_bytes                        # S = L*H*D*P
        self.S = (raw + self.G - 1) // self.G * self.G    # rounded up to a page-group multiple
        self.pool_total = pool_page_groups
        self.pool_free = pool_page_groups
        self.active = [False] * B
        self.mapped = [0] * B                             # page-groups mapped per sub-tensor
        self.map_calls = 0                                # cumulative (buffer, page) mappings
        self.unmap_calls = 0

    # ---- arithmetic -------------------------------------------------------------------------
    def need(self, seq_len: int) -> int:
        """Page-groups per sub-tensor that back seq_len tokens: (s + t - 1) / t, s = len*H*D*P."""
        s = seq_len * self.token_bytes
        return (s + self.G - 1) // self.G

    def va_offset(self, reqid: int) -> int:
        return reqid * self.S

    def tokens_per_page_group(self) -> int:
        return self.G // self.token_bytes

    # ---- Table 4 ----------------------------------------------------------------------------
    def alloc_reqid(self) -> int:
        free_ids = [r for r in range(self.B) if not self.active[r]]
        if not free_ids:
            return -1
        if self.policy == "deferred":
            r = max(free_ids, key=lambda x: (self.mapped[x], -x))
        else:
            r = free_ids[0]
        self.active[r] = True
        return r

    def free_reqid(self, reqid: int) -> int:
        if not (0 <= reqid < self.B) or not self.active[reqid]:
            return -1
        self.active[reqid] = False
        if self.policy == "sync":
            self._unmap_down_to(reqid, 0)
        return 0

    def step(self, seq_lens: Sequence[int]) -> int:
        if len(seq_lens) != self.B:
            return -1
        want = [0] * self.B
        for r in range(self.B):
            n = int(seq_lens[r])
            if n < 0 or n > self.L:
                return -1
            if not self.active[r]:
                if n != 0:
                    return -1
                continue
            want[r] = max(self.mapped[r], self.need(n))
        demand = sum(want[r] - self.mapped[r] for r in range(self.B) if self.active[r]) * self.nbuf
        reclaimable = sum(self.mapped[r] for r in range(self.B) if not self.active[r]) * self.nbuf
        if demand > self.pool_free + reclaimable:
            return -1
        if demand > self.pool_free:  # only reachable under "deferred"
            for r in range(self.B):
                if self.active[r]:
                    continue
                while self.mapped[r] > 0 and self.pool_free < demand:
                    self._unmap_down_to(r, self.mapped[r] - 1)
                if self.pool_free >= demand:
                    break
        for r in range(self.B):
            if self.active[r] and want[r] > self.mapped[r]:
                grow = want[r] - self.mapped[r]
                self.pool_free -= grow * self.nbuf
                self.map_calls += grow * self.nbuf
                self.sync_map_calls += grow * self.nbuf
                self.mapped[r] = want[r]
        if self.background:
            self._background_pass(seq_lens)
        return 0

    def next_candidate(self) -> int:
        """The id alloc_reqid would return now (-1 if none), without allocating it."""
        free_ids = [r for r in range(self.B) if not self.active[r]]
        if not free_ids:
            return -1
        if self.policy == "deferred":
            return max(free_ids, key=lambda x: (self.mapped[x], -x))
        return free_ids[0]

    def _grow(self, r: int, rows: int) -> None:
        self.pool_free -= rows * self.nbuf
        self.map_calls += rows * self.nbuf
        self.background_map_calls += rows * self.nbuf
        self.mapped[r] += rows

    def _background_pass(self, seq_lens: Sequence[int]) -> None:
        for r in range(self.B):                                   # 1. look-ahead
            n = int(seq_lens[r])
            if not self.active[r] or n == 0:
                continue
            grow = self.need(min(n + self.lookahead_tokens, self.L)) - self.mapped[r]
            if grow > 0 and grow * self.nbuf <= self.pool_free:
                self._grow(r, grow)
        if self.policy != "deferred":
            return
        cand = self.next_candidate()
        if self.pool_free < self.reclaim_threshold:               # 2. threshold reclamation
            for r in range(self.B):
                if self.active[r] or r == cand:
                    continue
                while self.mapped[r] > 0 and self.pool_free < self.reclaim_threshold:
                    self._unmap_down_to(r, self.mapped[r] - 1)
        if cand >= 0 and self.eager_page_groups > self.mapped[cand]:   # 3. eager allocation
            grow = min(self.eager_page_groups - self.mapped[cand], self.pool_free // self.nbuf)
            if grow > 0:
                self._grow(cand, grow)

    # ---- introspection ----------------------------------------------------------------------
    def query(self, reqid: int) -> Tuple[int, int, int]:
        """(active flag, page-groups mapped per sub-tensor, byte offset of the sub-tensor)."""
        return (1 if self.active[reqid] else 0, self.mapped[reqid], self.va_offset(reqid))

    def stats(self) -> Tuple[int, int, int, int]:
        return (self.G, self.S, self.pool_total, self.pool_free)

    def mapped_extents(self, reqid: int) -> List[Tuple[int, int]]:
        """Byte ranges [start, end) inside one buffer that are backed for this reqId."""
        base = self.va_offset(reqid)
        return [(base + k * self.G, base + (k + 1) * self.G) for k in range(self.mapped[reqid])]

    # ---- internals --------------------------------------------------------------------------
    def _unmap_down_to(self, reqid: int, keep: int) -> None:
        drop = self.mapped[reqid] - keep
        if drop > 0:
            self.pool_free += drop * self.nbuf
            self.unmap_calls += drop * self.nbuf
            self.mapped[reqid] = keep
