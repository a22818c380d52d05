"""Oracle: step-by-step simulation of the ODMA allocator (test infrastructure only).

The paper outlines the policy (Section III) without pseudo-code; this file
takes its steps in the paper's order and notation.  Where the paper is silent
the reading taken is stated next to the step.

State
    boundaries  b_1 < ... < b_B in tokens (Eq. 2), multiples of ``align``.
    two arenas in ONE token address space so a single offset indexes the pool:
        main    [0, main_tokens)               -- bucket slabs
        safety  [main_tokens, main+safety)     -- the Large Bucket (Section III-D)
    per arena: address-sorted list of free extents (start, size).  The paper's
        "per-size free lists" (Section III-E) do not say what happens to freed
        blocks once boundaries move; the reading here is address-ordered first
        fit with coalescing, which reuses a freed block of any size.
    per request: (arena, offset, cap, len).

Steps
    inflate   L' = ceil(L_hat * (1 + gamma*u))                 Section III-B
    route     u > tau (strict) or need > b_B  -> Large Bucket  Section III-B, III-D
              else bucket i = min{i : b_i >= need}, cap = b_i   Section III-A
    reserve   lowest-address free extent with size >= cap; take its low end
    advance   len + n > cap -> overflow flag, len unchanged     Section III-D
    migrate   reserve(safety, large_cap); copy len tokens; release the old slab
              (allocate-and-copy, Section IV-C); a request already in the safety
              arena cannot migrate again: it has reached L_max
    release   return [off, off+cap) to its arena and coalesce   Section III-E
    recalibrate  b_i = Q_{p_i}(L) over a sliding window, from a histogram with
              ``align``-wide bins (Eq. 2, Section III-C); integer arithmetic:
              k_i = max(1, ceil(p_i * n)) with p_i = num/den, j = first bin whose
              cumulative count reaches k_i, b_i = (j+1)*align; then force strictly
              increasing by +align, then clamp from the top so b_B <= large_cap.
              New boundaries affect later assigns only (Section IV-C).
    utilization  sum KV_actual / sum KV_reserved over completed requests
              (Section V); a migrated request counts the capacity it held at
              completion (``util``) or both slabs (``util_both``).

Status codes mirror the library's: 0 OK, -1 INVALID_ARG, -2 NOMEM, -3 OVERFLOW,
-4 UNKNOWN_REQ.

Pins (tests/test_oracle_allocator.py): invariants after every call (disjoint,
aligned, in-arena slabs; conservation of tokens; sorted non-adjacent free
extents); a bitmap allocator as an independent second implementation of first
fit; the nearest-rank order statistic from a sort for the quantiles; the
hand-worked Tiny example; the utilization inequality against worst-case
pre-allocation.
"""
from __future__ import annotations

import math
from collections import deque
from typing import Dict, List, Optional, Sequence, Tuple

OK, INVALID_ARG, NOMEM, OVERFLOW, UNKNOWN_REQ = 0, -1, -2, -3, -4
ARENA_MAIN, ARENA_SAFETY = 0, 1

DEFAULT_QUANTILES = {
    3: ((1, 2), (9, 10), (99, 100)),
    4: ((1, 2), (4, 5), (19, 20), (99, 100)),
}


class Arena:
    """Address-ordered first-fit extent allocator with coalescing."""

    def __init__(self, base: int, size: int):
        self.base, self.size = base, size
        self.free: List[List[int]] = [[base, size]] if size > 0 else []

    def reserve(self, cap: int) -> Optional[int]:
        for i, (start, size) in enumerate(self.free):
            if size >= cap:
                if size == cap:
                    del self.free[i]
                else:
                    self.free[i] = [start + cap, size - cap]
                return start
        return None

    def release(self, off: int, cap: int) -> None:
        i = 0
        while i < len(self.free) and self.free[i][0] < off:
            i += 1
        self.free.insert(i, [off, cap])
        if i + 1 < len(self.free) and self.free[i][0] + self.free[i][1] == self.free[i + 1][0]:
            self.free[i][1] += self.free[i + 1][1]
            del self.free[i + 1]
        if i > 0 and self.free[i - 1][0] + self.free[i - 1][1] == self.free[i][0]:
            self.free[i - 1][1] += self.free[i][1]
            del self.free[i]

    def free_tokens(self) -> int:
        return sum(s for _, s in self.free)


class PoolSim:
    def __init__(self, main_tokens: int, safety_tokens: int, large_cap: int, *, align: int = 16,
                 max_requests: int = 1 << 20, gamma: float = 0.2, tau: float = 0.8,
                 window: int = 10000, quantiles: Optional[Sequence[Tuple[int, int]]] = None,
                 boundaries: Sequence[int] = (512, 1024, 2048, 4096)):
        if align <= 0 or main_tokens % align or safety_tokens % align or large_cap % align or large_cap <= 0:
            raise ValueError("arena sizes and large_cap must be positive multiples of align")
        self.align, self.large_cap, self.max_requests = align, large_cap, max_requests
        self.gamma, self.tau, self.window = float(gamma), float(tau), int(window)
        self.main_tokens, self.safety_tokens = main_tokens, safety_tokens
        self.arenas = [Arena(0, main_tokens), Arena(main_tokens, safety_tokens)]
        self.req: Dict[int, List[int]] = {}          # id -> [arena, off, cap, len]
        self.boundaries = self._check_boundaries(boundaries)
        # the paper gives B = 4 but not the levels p_i; defaults exist for B = 3 and 4 only
        self.quantiles = tuple(quantiles) if quantiles is not None else DEFAULT_QUANTILES.get(len(self.boundaries))
        if self.quantiles is not None and len(self.quantiles) != len(self.boundaries):
            raise ValueError("one quantile level per bucket")
        self.ring: deque = deque()
        self.hist = [0] * (large_cap // align)
        # counters
        self.n_migrations = 0
        self.n_nomem = 0
        self.n_recalibrations = 0
        self.done_actual = 0        # sum of final lengths of released requests
        self.done_reserved = 0      # sum of capacity held at release
        self.done_reserved_both = 0  # ... plus capacities of slabs left by migration
        self._extra_reserved: Dict[int, int] = {}
        self._held: Dict[int, tuple] = {}   # source slabs of migrations whose release was deferred

    # -- helpers ---------------------------------------------------------------
    def _check_boundaries(self, b: Sequence[int]) -> Tuple[int, ...]:
        b = tuple(int(x) for x in b)
        if not b:
            raise ValueError("no boundaries")
        prev = 0
        for x in b:
            if x <= prev or x % self.align or x > self.large_cap:
                raise ValueError("boundaries must be increasing multiples of align, <= large_cap")
            prev = x
        return b

    def inflate(self, pred_len: int, u: float) -> int:
        """L' = ceil(L_hat * (1 + gamma*u)) in IEEE double."""
        return int(math.ceil(float(pred_len) * (1.0 + self.gamma * float(u))))

    # -- assignment ------------------------------------------------------------
    def assign(self, req_ids: Sequence[int], pred_len: Sequence[int],
               uncertainty: Optional[Sequence[float]] = None,
               prompt_len: Optional[Sequence[int]] = None,
               boundaries: Optional[Sequence[int]] = None):
        """Process requests in array order.  Returns lists (bucket, offset, cap, status).

        need = prompt + inflate(pred, u); bucket index B means the Large Bucket.
        A failed request leaves the pool unchanged and reports bucket -1,
        offset -1, cap 0.
        """
        b = self.boundaries if boundaries is None else self._check_boundaries(boundaries)
        nb = len(b)
        bucket, offset, cap, status = [], [], [], []
        for i, rid in enumerate(req_ids):
            rid = int(rid)
            u = 0.0 if uncertainty is None else float(uncertainty[i])
            prompt = 0 if prompt_len is None else int(prompt_len[i])
            pred = int(pred_len[i])
            st, bk, off, cp = OK, -1, -1, 0
            if rid < 0 or rid >= self.max_requests or pred < 0 or prompt < 0 or not (0.0 <= u <= 1.0):
                st = INVALID_ARG
            elif rid in self.req:
                st = UNKNOWN_REQ
            else:
                need = prompt + (self.inflate(pred, u) if uncertainty is not None else pred)
                need = max(need, 1)
                if need > self.large_cap:
                    st = OVERFLOW
                else:
                    if u > self.tau or need > b[-1]:
                        bk, cp, arena = nb, self.large_cap, ARENA_SAFETY
                    else:
                        bk = next(j for j in range(nb) if b[j] >= need)
                        cp, arena = b[bk], ARENA_MAIN
                    got = self.arenas[arena].reserve(cp)
                    if got is None:
                        st, bk, cp = NOMEM, -1, 0
                        self.n_nomem += 1
                    else:
                        off = got
                        self.req[rid] = [arena, off, cp, 0]
            bucket.append(bk); offset.append(off); cap.append(cp); status.append(st)
        return bucket, offset, cap, status

    # -- decode-time bookkeeping --------------------------------------------------
    def advance(self, req_ids: Sequence[int], n_new: Optional[Sequence[int]] = None):
        """len += n unless that would exceed cap.  Returns (overflow flags, status)."""
        overflow, status = [], []
        for i, rid in enumerate(req_ids):
            rid = int(rid)
            n = 1 if n_new is None else int(n_new[i])
            rec = self.req.get(rid)
            if rec is None:
                overflow.append(0); status.append(UNKNOWN_REQ)
            elif n < 0:
                overflow.append(0); status.append(INVALID_ARG)
            elif rec[3] + n > rec[2]:
                overflow.append(1); status.append(OK)
            else:
                rec[3] += n
                overflow.append(0); status.append(OK)
        return overflow, status

    def migrate(self, rid: int, defer_release: bool = False):
        """Returns (status, new_offset, new_cap, old_offset, len_copied).

        With defer_release the source slab stays reserved until finish_migration
        (the copy may then run beside other work that could otherwise reuse it)."""
        rec = self.req.get(int(rid))
        if rec is None:
            return UNKNOWN_REQ, -1, 0, -1, 0
        arena, off, cap, ln = rec
        if arena == ARENA_SAFETY:
            return OVERFLOW, -1, 0, -1, 0
        new_off = self.arenas[ARENA_SAFETY].reserve(self.large_cap)
        if new_off is None:
            self.n_nomem += 1
            return NOMEM, -1, 0, -1, 0
        if defer_release:
            self._held[int(rid)] = (arena, off, cap)
        else:
            self.arenas[arena].release(off, cap)
        self.req[int(rid)] = [ARENA_SAFETY, new_off, self.large_cap, ln]
        self._extra_reserved[int(rid)] = self._extra_reserved.get(int(rid), 0) + cap
        self.n_migrations += 1
        return OK, new_off, self.large_cap, off, ln

    def finish_migration(self, req_ids: Sequence[int]):
        """Releases source slabs kept by migrate(defer_release=True)."""
        status = []
        for rid in req_ids:
            held = self._held.pop(int(rid), None) if int(rid) in self.req else None
            if held is None:
                status.append(UNKNOWN_REQ)
                continue
            self.arenas[held[0]].release(held[1], held[2])
            status.append(OK)
        return status

    def release(self, req_ids: Sequence[int]):
        status = []
        for rid in req_ids:
            rid = int(rid)
            rec = self.req.pop(rid, None)
            if rec is None:
                status.append(UNKNOWN_REQ)
                continue
            arena, off, cap, ln = rec
            self.arenas[arena].release(off, cap)
            held = self._held.pop(rid, None)
            if held is not None:
                self.arenas[held[0]].release(held[1], held[2])
            self.done_actual += ln
            self.done_reserved += cap
            self.done_reserved_both += cap + self._extra_reserved.pop(rid, 0)
            status.append(OK)
        return status

    # -- adaptive bucket manager ---------------------------------------------------
    def recalibrate(self, realized: Sequence[int] = ()):
        """Push realized lengths into the window, then re-derive the boundaries."""
        if self.quantiles is None:
            raise ValueError("no quantile levels configured for this number of buckets")
        w = self.align
        for L in realized:
            L = min(max(int(L), 1), self.large_cap)
            if len(self.ring) == self.window:
                old = self.ring.popleft()
                self.hist[(old - 1) // w] -= 1
            self.ring.append(L)
            self.hist[(L - 1) // w] += 1
        n = len(self.ring)
        if n == 0:
            return self.boundaries
        b = []
        for num, den in self.quantiles:
            k = max(1, (num * n + den - 1) // den)
            cum, j = 0, 0
            for j, c in enumerate(self.hist):
                cum += c
                if cum >= k:
                    break
            b.append((j + 1) * w)
        for i in range(1, len(b)):
            b[i] = max(b[i], b[i - 1] + w)
        b[-1] = min(b[-1], self.large_cap)
        for i in range(len(b) - 2, -1, -1):
            b[i] = min(b[i], b[i + 1] - w)
        self.boundaries = tuple(b)
        self.n_recalibrations += 1
        return self.boundaries

    # -- introspection ----------------------------------------------------------------
    def snapshot(self):
        """Live requests sorted by id: list of (id, arena, offset, cap, len)."""
        return [(rid, *self.req[rid]) for rid in sorted(self.req)]

    def held_slabs(self):
        """Source slabs of deferred migrations: {request id: (arena, offset, cap)}."""
        return dict(self._held)

    def free_extents(self, arena: int):
        return [tuple(e) for e in self.arenas[arena].free]

    def utilization(self) -> float:
        return self.done_actual / self.done_reserved if self.done_reserved else 0.0

    def utilization_both(self) -> float:
        return self.done_actual / self.done_reserved_both if self.done_reserved_both else 0.0
