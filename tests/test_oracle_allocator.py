"""Pins for oracle/allocator.py: invariants, an independent bitmap first-fit,
sorted-order quantiles, the hand-worked Tiny example, the utilization bound."""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import allocator as al

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# P7: invariants that must hold after every call
# ---------------------------------------------------------------------------

def check_invariants(sim: al.PoolSim, caps_allowed=None):
    snap = sim.snapshot()
    spans = {0: [], 1: []}
    for rid, arena, off, cap, ln in snap:
        base, size = sim.arenas[arena].base, sim.arenas[arena].size
        assert base <= off and off + cap <= base + size, "slab outside its arena"
        assert off % sim.align == 0 and cap % sim.align == 0
        assert 0 <= ln <= cap
        if arena == al.ARENA_SAFETY:
            assert cap == sim.large_cap
        elif caps_allowed is not None:
            assert cap in caps_allowed
        spans[arena].append((off, off + cap))
    for rid, (arena, off, cap) in sim.held_slabs().items():          # sources of deferred migrations stay reserved
        assert rid in {t[0] for t in snap}
        spans[arena].append((off, off + cap))
    for arena in (0, 1):
        a = sim.arenas[arena]
        free = sim.free_extents(arena)
        for (s0, n0), (s1, n1) in zip(free[:-1], free[1:]):
            assert s0 + n0 < s1, "free extents must be sorted and non-adjacent"
        for s, n in free:
            assert n > 0 and a.base <= s and s + n <= a.base + a.size
        everything = sorted(spans[arena] + [(s, s + n) for s, n in free])
        pos = a.base
        for lo, hi in everything:
            assert lo == pos, "overlap or hole between slabs and free extents"
            pos = hi
        assert pos == a.base + a.size
        assert sum(hi - lo for lo, hi in spans[arena]) + a.free_tokens() == a.size


# ---------------------------------------------------------------------------
# P8: independent second implementation of address-ordered first fit
# ---------------------------------------------------------------------------

class BitmapArena:
    def __init__(self, base, size):
        self.base, self.used = base, np.zeros(size, dtype=bool)

    def reserve(self, cap):
        run = 0
        for i, u in enumerate(self.used):
            run = 0 if u else run + 1
            if run == cap:
                start = i - cap + 1
                self.used[start:i + 1] = True
                return self.base + start
        return None

    def release(self, off, cap):
        assert self.used[off - self.base: off - self.base + cap].all()
        self.used[off - self.base: off - self.base + cap] = False


@pytest.mark.parametrize("seed", range(8))
def test_random_trace_matches_bitmap_allocator_and_keeps_invariants(seed):
    rng = np.random.default_rng(seed)
    align = 16
    bounds = (32, 64, 128, 256)
    sim = al.PoolSim(2048, 1024, 512, align=align, boundaries=bounds, max_requests=64)
    bm = [BitmapArena(0, 2048), BitmapArena(2048, 1024)]
    live, held = {}, {}
    for step in range(600):
        op = rng.choice(["assign", "assign", "release", "advance", "migrate", "migrate_deferred", "finish"])
        if op == "assign":
            rid = int(rng.integers(0, 64))
            pred = int(rng.integers(1, 400))
            u = float(np.float32(rng.random()))
            bk, off, cap, st = sim.assign([rid], [pred], [u])
            if rid in live:
                assert st[0] == al.UNKNOWN_REQ
            else:
                need = sim.inflate(pred, u)
                if u > 0.8 or need > bounds[-1]:
                    want_cap, arena = 512, 1
                else:
                    want_cap, arena = min(b for b in bounds if b >= need), 0
                expect = bm[arena].reserve(want_cap)
                if expect is None:
                    assert st[0] == al.NOMEM and off[0] == -1
                else:
                    assert st[0] == al.OK and off[0] == expect and cap[0] == want_cap
                    assert bk[0] == (4 if arena else bounds.index(want_cap))
                    live[rid] = [arena, expect, want_cap, 0]
        elif op == "release" and live:
            rid = int(rng.choice(list(live)))
            assert sim.release([rid]) == [al.OK]
            arena, off, cap, _ = live.pop(rid)
            bm[arena].release(off, cap)
            if rid in held:                                              # a source still held goes with its request
                bm[held[rid][0]].release(*held.pop(rid)[1:])
            assert sim.release([rid]) == [al.UNKNOWN_REQ]
        elif op == "advance" and live:
            rid = int(rng.choice(list(live)))
            n = int(rng.integers(1, 80))
            ov, st = sim.advance([rid], [n])
            rec = live[rid]
            if rec[3] + n > rec[2]:
                assert ov == [1]
            else:
                assert ov == [0]; rec[3] += n
        elif op in ("migrate", "migrate_deferred") and live:
            rid = int(rng.choice(list(live)))
            rec = live[rid]
            defer = op == "migrate_deferred"
            st, noff, ncap, ooff, ln = sim.migrate(rid, defer_release=defer)
            if rec[0] == 1:
                assert st == al.OVERFLOW
            else:
                expect = bm[1].reserve(512)
                if expect is None:
                    assert st == al.NOMEM
                else:
                    assert (st, noff, ncap, ooff, ln) == (al.OK, expect, 512, rec[1], rec[3])
                    if defer:
                        held[rid] = (0, rec[1], rec[2])                  # the source stays reserved until finish
                    else:
                        bm[0].release(rec[1], rec[2])
                    live[rid] = [1, expect, 512, rec[3]]
        elif op == "finish":
            rid = int(rng.integers(0, 64))
            st = sim.finish_migration([rid])
            if rid in held:
                assert st == [al.OK]
                bm[held[rid][0]].release(*held.pop(rid)[1:])
            else:
                assert st == [al.UNKNOWN_REQ]
        assert sim.held_slabs() == held
        check_invariants(sim, caps_allowed=set(bounds))
        assert {t[0]: tuple(t[1:]) for t in sim.snapshot()} == {r: tuple(v) for r, v in live.items()}
    sim.release(list(live))
    assert sim.free_extents(0) == [(0, 2048)] and sim.free_extents(1) == [(2048, 1024)]


# ---------------------------------------------------------------------------
# P9: hand-worked Tiny example (derived by hand from the reading of Sections
# III-A, III-D and V; the paper itself prints no worked example)
# ---------------------------------------------------------------------------

def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([int(x) for x in line.split()])
    return rows


def test_tiny_worked_example_perfect_prediction():
    w = wl.tiny()
    lens = w.lengths.tolist()
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries,
                     quantiles=al.DEFAULT_QUANTILES[3])
    bk, off, cap, st = sim.assign(range(4), lens)
    gold = _read_golden("tiny_perfect_prediction.txt")
    assert [[r, lens[r], bk[r], off[r], cap[r]] for r in range(4)] == gold
    assert st == [0, 0, 0, 0]
    sim.advance(range(4), lens)
    sim.release(range(4))
    assert sim.done_actual == 366 and sim.done_reserved == 512
    assert abs(sim.utilization() - 366 / 512) < 1e-15
    # static worst-case pre-allocation reserves L_max = 256 for each of the 4 requests
    assert abs(366 / (4 * w.large_cap) - 0.357421875) < 1e-15


def test_tiny_worked_example_underprediction_migrates():
    w = wl.tiny()
    lens = w.lengths.tolist()
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries,
                     quantiles=al.DEFAULT_QUANTILES[3])
    pred = [60] + lens[1:]
    bk, off, cap, st = sim.assign(range(4), pred)
    gold = _read_golden("tiny_underprediction.txt")
    assert [[r, pred[r], bk[r], off[r], cap[r]] for r in range(4)] == gold[:4]
    assert sim.advance([0], [64]) == ([0], [0])
    assert sim.advance([0], [1]) == ([1], [0])              # the 65th token overflows
    st, noff, ncap, ooff, ln = sim.migrate(0)
    assert [st, noff, ncap, ooff, ln] == gold[4]
    assert sim.free_extents(0)[0] == (0, 64)                 # the old slab is free again
    assert sim.advance([0], [1]) == ([0], [0])
    assert sim.migrate(0)[0] == al.OVERFLOW                  # already in the Large Bucket
    check_invariants(sim)


# ---------------------------------------------------------------------------
# routing rules (Section III-B, III-D)
# ---------------------------------------------------------------------------

def test_inflation_and_routing():
    sim = al.PoolSim(4096, 2048, 1024, boundaries=(64, 128, 256, 512))
    assert sim.inflate(100, 0.0) == 100
    # IEEE double: 1 + 0.2*0.5 rounds to 1.100000000000000089 and 100x that to 110.00000000000001,
    # so the ceiling is 111 (the reading errs on the side of reserving more)
    assert sim.inflate(100, 0.5) == 111
    exact = al.PoolSim(4096, 2048, 1024, boundaries=(64, 128, 256, 512), gamma=0.25)
    assert exact.inflate(64, 0.5) == 72 and exact.inflate(100, 0.5) == 113 and exact.inflate(7, 1.0) == 9
    assert sim.inflate(100, 1.0) == 120
    assert sim.inflate(101, 0.5) == 112          # ceil(111.1)
    bk, off, cap, st = sim.assign([0, 1, 2, 3, 4, 5], [64, 65, 100, 100, 513, 1025],
                                  [0.0, 0.0, 0.8, np.float32(0.81), 0.0, 0.0])
    assert bk == [0, 1, 1, 4, 4, -1]             # == boundary fits; u = tau stays; u > tau routed; > b_B routed
    assert cap == [64, 128, 128, 1024, 1024, 0]
    assert st == [0, 0, 0, 0, 0, al.OVERFLOW]
    assert off[3] == 4096 and off[4] == 4096 + 1024
    # prompt tokens are added after inflating the predicted generation length
    bk, off, cap, st = sim.assign([6], [100], [0.5], prompt_len=[19])
    assert cap == [256] and bk == [2]            # 19 + 110 = 129 > 128
    # safety pool exhausted -> NOMEM and nothing changes
    before = sim.snapshot()
    assert sim.assign([7], [600])[3] == [al.NOMEM]
    assert sim.snapshot() == before and sim.n_nomem == 1
    # no spill of a bucket request into the safety pool or a larger bucket when main is full
    sim2 = al.PoolSim(128, 1024, 512, boundaries=(64, 128))
    assert sim2.assign([0, 1, 2], [64, 64, 10])[3] == [0, 0, al.NOMEM]


def test_boundaries_passed_to_assign_do_not_touch_live_requests():
    sim = al.PoolSim(4096, 1024, 1024, boundaries=(64, 128, 256, 512))
    sim.assign([0], [100])
    sim.assign([1], [100], boundaries=(112, 256, 512, 1024))
    snap = dict((r[0], r) for r in sim.snapshot())
    assert snap[0][3] == 128 and snap[1][3] == 112
    with pytest.raises(ValueError):
        sim.assign([2], [5], boundaries=(64, 64, 128, 256))


# ---------------------------------------------------------------------------
# P10: quantile recalibration (Eq. 2)
# ---------------------------------------------------------------------------

def _ref_boundaries(window, quantiles, w, large_cap):
    s = sorted(min(max(int(x), 1), large_cap) for x in window)
    n = len(s)
    b = []
    for num, den in quantiles:
        k = max(1, -(-num * n // den))
        b.append(-(-s[k - 1] // w) * w)
    for i in range(1, len(b)):
        b[i] = max(b[i], b[i - 1] + w)
    b[-1] = min(b[-1], large_cap)
    for i in range(len(b) - 2, -1, -1):
        b[i] = min(b[i], b[i + 1] - w)
    return tuple(b)


@pytest.mark.parametrize("seed", range(6))
def test_recalibration_equals_rounded_order_statistic(seed):
    rng = np.random.default_rng(seed)
    W = 500
    sim = al.PoolSim(1 << 16, 1 << 16, 8192, window=W, boundaries=(512, 1024, 2048, 4096))
    hist = []
    for _ in range(12):
        batch = wl.pareto(rng, int(rng.integers(1, 200)), 1.3, 8, 20000).tolist()
        hist += batch
        got = sim.recalibrate(batch)
        assert got == _ref_boundaries(hist[-W:], al.DEFAULT_QUANTILES[4], 16, 8192)
        assert sim.recalibrate([]) == got                      # idempotent on an unchanged window
        assert all(a < b for a, b in zip(got[:-1], got[1:])) and got[-1] <= 8192
        assert all(x % 16 == 0 for x in got)


def test_recalibration_closed_form_uniform_and_eviction():
    N = 1000
    sim = al.PoolSim(1 << 16, 1 << 16, 4096, window=N, boundaries=(512, 1024, 2048, 4096))
    got = sim.recalibrate(range(1, N + 1))
    # lengths 1..N: the k-th order statistic is k = ceil(p N)
    want = tuple(-(-(-(-num * N // den)) // 16) * 16 for num, den in al.DEFAULT_QUANTILES[4])
    assert got == want == (512, 800, 960, 992)
    # after W identical new samples the old distribution has no influence
    got = sim.recalibrate([100] * N)
    assert got == (112, 128, 144, 160)          # all quantiles in bin 96<L<=112, forced apart by +16
    assert sum(sim.hist) == N and sim.hist[(100 - 1) // 16] == N
    # empty window leaves boundaries unchanged
    sim2 = al.PoolSim(4096, 4096, 4096, boundaries=(64, 128, 256, 512))
    assert sim2.recalibrate([]) == (64, 128, 256, 512) and sim2.n_recalibrations == 0
    # clamp from the top keeps them strictly increasing and <= large_cap
    sim3 = al.PoolSim(4096, 4096, 64, boundaries=(16, 32, 48, 64))
    assert sim3.recalibrate([64] * 10) == (16, 32, 48, 64)
    assert sim3.recalibrate([10 ** 6] * 10) == (16, 32, 48, 64)   # clamped into [1, large_cap]


# ---------------------------------------------------------------------------
# P11: utilization never below worst-case pre-allocation; closed form
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(4))
def test_utilization_bound_and_closed_form(seed):
    rng = np.random.default_rng(seed)
    lens = wl.lognorm(rng, 300, 512, 0.8, 1, 4096)
    bounds = (1024, 2048, 4096)
    sim = al.PoolSim(300 * 4096, 8 * 4096, 4096, boundaries=bounds, quantiles=al.DEFAULT_QUANTILES[3])
    _, _, cap, st = sim.assign(range(300), lens.tolist())
    assert set(st) == {0}
    sim.advance(range(300), lens.tolist())
    sim.release(range(300))
    want = lens.sum() / sum(min(b for b in bounds if b >= x) for x in lens)
    assert abs(sim.utilization() - want) < 1e-15
    static = lens.sum() / (300 * 4096)
    assert sim.utilization() >= static
    assert sim.utilization_both() == sim.utilization()        # nothing migrated


def test_config2_utilization_figures():
    """The seeded batch-64 config: utilization 0.529 against 0.178 for worst-case reservation."""
    w = wl.qwen_b64()
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries,
                     quantiles=al.DEFAULT_QUANTILES[3])
    sim.assign(range(64), w.lengths.tolist())
    sim.advance(range(64), w.lengths.tolist())
    check_invariants(sim, set(w.boundaries))
    sim.release(range(64))
    assert round(sim.utilization(), 3) == 0.529
    assert round(w.lengths.sum() / (64 * 4096), 3) == 0.178


def test_migrated_request_utilization_variants():
    sim = al.PoolSim(1024, 512, 256, boundaries=(64, 128))
    sim.assign([0], [64]); sim.advance([0], [64])
    assert sim.migrate(0)[0] == al.OK
    sim.advance([0], [36]); sim.release([0])
    assert sim.utilization() == 100 / 256 and sim.utilization_both() == 100 / (256 + 64)
    assert sim.n_migrations == 1
