"""Host side of libodma against the allocator oracle: bit-exact on every output.

Runs without a GPU (the library's host calls never touch the device)."""
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import allocator as al
from paper_2512_09427_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def make_pair(main, safety, large_cap, bounds, *, max_requests=64, window=10000, quantiles=None, gamma=0.2, tau=0.8,
              align=16):
    cfg, keep = B.make_config(n_layers=1, n_q_heads=2, n_kv_heads=1, head_dim=64, kv_dtype=B.F32, out_dtype=B.F32,
                              main_tokens=main, safety_tokens=safety, large_cap=large_cap, boundaries=bounds,
                              max_requests=max_requests, window=window, quantiles=quantiles, gamma=gamma, tau=tau,
                              align_tokens=align)
    pool = B.Pool(cfg, keep)
    sim = al.PoolSim(main, safety, large_cap, align=align, max_requests=max_requests, gamma=gamma, tau=tau,
                     window=window, quantiles=quantiles, boundaries=bounds)
    return pool, sim


def assert_same_state(pool: B.Pool, sim: al.PoolSim):
    rows, bounds = pool.odma_pool_snapshot()
    assert rows == [tuple(r) for r in sim.snapshot()]
    assert bounds == tuple(sim.boundaries)
    for arena in (0, 1):
        assert pool.odma_pool_free_extents(arena) == sim.free_extents(arena)
    st = pool.odma_pool_stats()
    assert st["migrations"] == sim.n_migrations and st["nomem"] == sim.n_nomem
    assert st["recalibrations"] == sim.n_recalibrations
    assert st["done_actual"] == sim.done_actual and st["done_reserved"] == sim.done_reserved
    assert st["done_reserved_both"] == sim.done_reserved_both
    assert st["live_requests"] == len(sim.req)
    assert st["live_tokens"] == sum(r[3] for r in sim.req.values())
    assert st["live_reserved"] == sum(r[2] for r in sim.req.values())


# ---- ABI surface ---------------------------------------------------------------------------

def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "odma.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(odma_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name
    assert "gfx950" in B.odma_version()


def test_invalid_configurations_are_rejected():
    good = dict(n_layers=1, n_q_heads=28, n_kv_heads=4, head_dim=128, kv_dtype=B.BF16, out_dtype=B.BF16,
                main_tokens=4096, safety_tokens=4096, large_cap=4096, boundaries=(1024, 2048, 4096), max_requests=8)
    B.Pool(*B.make_config(**good)).close()
    for bad in (dict(n_q_heads=30), dict(head_dim=100), dict(main_tokens=4100), dict(large_cap=1000),
                dict(boundaries=(2048, 1024, 4096)), dict(boundaries=(1024, 2048, 8192)), dict(max_requests=0),
                dict(kv_dtype=5), dict(n_kv_heads=1), dict(decode_kernel=B.KERNEL_MFMA, head_dim=32),
                dict(kv_dtype=B.FP8, head_dim=64), dict(kv_dtype=B.FP8, decode_kernel=B.KERNEL_VALU)):
        with pytest.raises(B.OdmaError):
            B.Pool(*B.make_config(**{**good, **bad}))
    cfg, keep = B.make_config(**good)
    assert B.odma_workspace_bytes(cfg) % 256 == 0
    # device calls on a pool without device memory fail cleanly
    p = B.Pool(cfg, keep)
    assert B.lib.odma_decode_attention(p._h, 0, 1, None, None, None, None, 0, None, 0, None) == B.INVALID_ARG
    assert "device memory" in B.odma_last_error()


# ---- randomized traces -----------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(10))
def test_random_trace_is_bit_exact(seed):
    rng = np.random.default_rng(seed)
    bounds = (32, 64, 128, 256)
    pool, sim = make_pair(2048, 1024, 512, bounds, max_requests=48, window=64)
    for step in range(300):
        op = rng.choice(["assign", "assign", "release", "advance", "migrate", "recal"])
        if op == "assign":
            k = int(rng.integers(1, 6))
            ids = rng.integers(-1, 50, k)                     # includes invalid and duplicate ids
            pred = rng.integers(-2, 600, k)
            u = rng.random(k).astype(np.float32) if rng.random() < 0.7 else None
            prompt = rng.integers(0, 40, k) if rng.random() < 0.5 else None
            b = None
            if rng.random() < 0.2:
                b = tuple(sorted(rng.choice(np.arange(16, 513, 16), 3, replace=False).tolist()))
            rc, bk, off, cap, st = pool.odma_assign(ids, pred, u, prompt, b)
            sbk, soff, scap, sst = sim.assign(ids.tolist(), pred.tolist(), None if u is None else u,
                                              None if prompt is None else prompt.tolist(), b)
            assert bk.tolist() == sbk and off.tolist() == soff and cap.tolist() == scap and st.tolist() == sst
            assert rc == next((s for s in sst if s), 0)
        elif op == "release":
            ids = rng.integers(0, 48, int(rng.integers(1, 4)))
            rc, st = pool.odma_release(ids)
            assert st.tolist() == sim.release(ids.tolist())
        elif op == "advance":
            ids = rng.integers(0, 48, int(rng.integers(1, 8)))
            nn = rng.integers(0, 70, len(ids)) if rng.random() < 0.7 else None
            rc, ov, st = pool.odma_advance(ids, nn)
            sov, sst = sim.advance(ids.tolist(), None if nn is None else nn.tolist())
            assert ov.tolist() == sov and st.tolist() == sst
        elif op == "migrate":
            rid = int(rng.integers(0, 48))
            rc, noff, ncap = pool.odma_migrate(rid)
            sst, snoff, sncap, _, _ = sim.migrate(rid)
            assert (rc, noff, ncap) == (sst, snoff, sncap)
        else:
            lens = wl.pareto(rng, int(rng.integers(0, 40)), 1.2, 4, 2000).tolist()
            assert pool.odma_recalibrate(lens) == tuple(sim.recalibrate(lens))
        assert_same_state(pool, sim)


def test_inflate_matches_oracle_on_many_inputs():
    pool, sim = make_pair(4096, 4096, 4096, (512, 1024, 2048, 4096))
    rng = np.random.default_rng(0)
    for _ in range(20000):
        L, u = int(rng.integers(0, 100000)), np.float32(rng.random())
        assert pool.odma_inflate(L, u) == sim.inflate(L, u)
    for L in (0, 1, 100, 101, 2 ** 31 - 1):
        for u in map(np.float32, (0.0, 0.5, 0.8, 1.0)):       # the ABI carries u as a float
            assert pool.odma_inflate(L, u) == sim.inflate(L, u)


# ---- the seeded configurations ---------------------------------------------------------------

def test_tiny_golden_example_through_the_library():
    w = wl.tiny()
    pool, _ = make_pair(w.main_tokens, w.safety_tokens, w.large_cap, w.boundaries)
    rc, bk, off, cap, st = pool.odma_assign(range(4), [60, 73, 101, 123])
    assert (rc, bk.tolist(), off.tolist(), cap.tolist()) == (0, [0, 1, 1, 1], [0, 64, 192, 320], [64, 128, 128, 128])
    assert pool.odma_advance([0], [64])[1].tolist() == [0]
    assert pool.odma_advance([0], [1])[1].tolist() == [1]
    assert pool.odma_migrate(0) == (0, 1024, 256)
    assert pool.odma_pool_free_extents(0)[0] == (0, 64)
    assert pool.odma_migrate(0)[0] == B.OVERFLOW
    assert pool.odma_migrate(9)[0] == B.UNKNOWN_REQ
    off, ln, cap = pool.odma_pool_lookup([0, 1])
    assert off.tolist() == [1024, 64] and ln.tolist() == [64, 0] and cap.tolist() == [256, 128]


@pytest.mark.parametrize("maker", [wl.qwen_b64, wl.qwen_b256_pareto, wl.qwen_b128_step])
def test_seeded_configs_assign_identically(maker):
    w = maker()
    n = w.n_requests
    pool, sim = make_pair(w.main_tokens, w.safety_tokens, w.large_cap, w.boundaries, max_requests=n)
    if w.name.endswith("pareto"):        # config 3: boundaries recalibrated on the batch itself
        assert pool.odma_recalibrate(w.lengths.tolist()) == tuple(sim.recalibrate(w.lengths.tolist()))
    steps = w.extra.get("steps", 0)
    pred = (w.lengths + steps).tolist()
    rc, bk, off, cap, st = pool.odma_assign(range(n), pred)
    sbk, soff, scap, sst = sim.assign(range(n), pred)
    assert rc == 0 and bk.tolist() == sbk and off.tolist() == soff and cap.tolist() == scap
    pool.odma_advance(range(n), w.lengths.tolist()); sim.advance(range(n), w.lengths.tolist())
    assert_same_state(pool, sim)
    pool.odma_release(range(n)); sim.release(range(n))
    assert_same_state(pool, sim)
    assert pool.odma_pool_free_extents(0) == [(0, w.main_tokens)]


def test_drift_run_bookkeeping_is_bit_exact():
    """Config 5's host loop (admit, decode, overflow -> migrate, complete, recalibrate) on a short horizon."""
    slots, steps = 48, 400
    bounds = (512, 1024, 2048, 4096)
    pool, sim = make_pair(1 << 18, 4 * 65536, 65536, bounds, max_requests=slots, window=256)
    gen = wl.drift_arrivals(seed=5, n_steps=steps)
    next(gen)
    live = {}
    done = []
    for step in range(steps):
        for s in range(slots):
            if s not in live:
                a = gen.send(step)
                args = ([s], [a.pred_len], np.array([a.uncertainty], np.float32))
                rc, bk, off, cap, st = pool.odma_assign(*args)
                sres = sim.assign([s], [a.pred_len], [np.float32(a.uncertainty)])
                assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(map(list, sres))
                if st[0] != 0:
                    continue
                # prefill; an under-predicted prompt may already overflow the bucket
                rc, ov, _ = pool.odma_advance([s], [a.prefilled]); sov, _ = sim.advance([s], [a.prefilled])
                assert ov.tolist() == sov
                if ov[0]:
                    assert pool.odma_migrate(s)[:2] == sim.migrate(s)[:2]
                    assert pool.odma_advance([s], [a.prefilled])[1].tolist() == sim.advance([s], [a.prefilled])[0]
                live[s] = [a.total_len, a.prefilled]
        ids = sorted(live)
        rc, ov, _ = pool.odma_advance(ids); sov, _ = sim.advance(ids)
        assert ov.tolist() == sov
        for s, o in zip(ids, ov):
            if o:
                got, want = pool.odma_migrate(s), sim.migrate(s)
                assert got == want[:3]
                if got[0] == 0:
                    pool.odma_advance([s]); sim.advance([s])
                    live[s][1] += 1
            else:
                live[s][1] += 1
        fin = [s for s in ids if live[s][1] >= live[s][0]]
        if fin:
            done += [live[s][0] for s in fin]
            assert pool.odma_release(fin)[1].tolist() == sim.release(fin)
            for s in fin:
                del live[s]
        if step % 50 == 49:
            assert pool.odma_recalibrate(done) == tuple(sim.recalibrate(done))
            done = []
        if step % 20 == 0:
            assert_same_state(pool, sim)
    assert_same_state(pool, sim)
    assert sim.n_recalibrations >= 7 and sim.done_actual > 0


def test_failure_paths_leave_state_untouched():
    pool, sim = make_pair(256, 512, 512, (64, 128), max_requests=8)
    assert pool.odma_assign([0, 1, 2], [128, 128, 1])[4].tolist() == [0, 0, B.NOMEM]      # main arena full
    assert pool.odma_assign([3, 4], [300, 300])[4].tolist() == [0, B.NOMEM]                # safety full
    rows, _ = pool.odma_pool_snapshot()
    assert pool.odma_migrate(0)[0] == B.NOMEM                                               # request stays intact
    assert pool.odma_pool_snapshot()[0] == rows
    assert pool.odma_advance([0], [129])[1].tolist() == [1]                                 # overflow, len unchanged
    assert pool.odma_pool_lookup([0])[1].tolist() == [0]
    assert pool.odma_release([5])[0] == B.UNKNOWN_REQ
    assert pool.odma_release([0])[0] == 0 and pool.odma_release([0])[0] == B.UNKNOWN_REQ    # double release
    assert pool.odma_assign([1], [10])[4].tolist() == [B.UNKNOWN_REQ]                       # duplicate live id
    assert pool.odma_assign([6], [513])[4].tolist() == [B.OVERFLOW]                         # beyond L_max
    assert pool.odma_assign([6], [5], boundaries=(128, 64))[0] == B.INVALID_ARG
    assert pool.odma_pool_stats()["nomem"] == 3


def test_tune_knobs_accept_documented_ranges_only():
    """odma_pool_tune is host-side state: every knob takes its documented range and rejects the rest."""
    pool, _ = make_pair(256, 512, 512, (64, 128), max_requests=8)
    ranges = {B.TUNE_WAVES_PER_CU: ((0, 1, 8, 64), (-1, 65)), B.TUNE_ITEMS_PER_WAVE: ((4, 32, 256), (3, 257)),
              B.TUNE_MIN_CHUNK: ((64, 128, 4096), (0, 32, 100)), B.TUNE_PIPELINE_DEPTH: ((2, 3), (1, 4)),
              B.TUNE_WAVES_PER_WG: ((0, 4, 8), (2, 6, 16)), B.TUNE_ODD_XCD_WEIGHT: ((128, 256, 512), (127, 513)),
              B.TUNE_LATE_WAVE_WEIGHT: ((128, 256, 512), (127, 513)), B.TUNE_FUSE_REDUCE: ((0, 1), (-1, 2))}
    for knob, (good, bad) in ranges.items():
        for v in good:
            assert pool.odma_pool_tune(knob, v) == 0, (knob, v)
        for v in bad:
            with pytest.raises(B.OdmaError) as e:
                pool.odma_pool_tune(knob, v)
            assert e.value.code == B.INVALID_ARG, (knob, v)
    with pytest.raises(B.OdmaError):
        pool.odma_pool_tune(99, 1)


def test_batched_migration_and_deferred_release_are_bit_exact():
    """odma_migrate_batch == the oracle's migrate in array order; deferred sources stay reserved until finish."""
    pool, sim = make_pair(1 << 14, 6 * 2048, 2048, (256, 512, 1024), max_requests=32)
    rng = np.random.default_rng(3)
    lens = [int(x) for x in rng.integers(10, 900, 20)]
    ids = list(range(20))
    pool.odma_assign(ids, lens); sim.assign(ids, lens)
    pool.odma_advance(ids, lens); sim.advance(ids, lens)
    # immediate release: three requests, one unknown id in the middle
    rc, off, cap, st = pool.odma_migrate_batch([3, 25, 7, 11])
    want = [sim.migrate(r) for r in (3, 25, 7, 11)]
    assert st.tolist() == [w[0] for w in want] == [0, B.UNKNOWN_REQ, 0, 0] and rc == B.UNKNOWN_REQ
    assert off.tolist() == [w[1] for w in want] and cap.tolist() == [w[2] for w in want]
    assert_same_state(pool, sim)
    # deferred release: sources stay reserved, a new admission cannot take them
    rc, off, cap, st = pool.odma_migrate_batch([1, 2, 3], B.MIGRATE_DEFER_RELEASE)      # 3 already sits in the Large Bucket
    want = [sim.migrate(r, defer_release=True) for r in (1, 2, 3)]
    assert st.tolist() == [w[0] for w in want] == [0, 0, B.OVERFLOW]
    assert off.tolist() == [w[1] for w in want]
    assert_same_state(pool, sim)
    got = pool.odma_assign([20, 21], [900, 200]); exp = sim.assign([20, 21], [900, 200])
    assert (got[1].tolist(), got[2].tolist(), got[3].tolist(), got[4].tolist()) == tuple(map(list, exp))
    assert pool.odma_migrate_finish([1, 9, 2])[1].tolist() == sim.finish_migration([1, 9, 2]) == [0, B.UNKNOWN_REQ, 0]
    assert pool.odma_migrate_finish([1])[1].tolist() == sim.finish_migration([1]) == [B.UNKNOWN_REQ]   # nothing held any more
    assert_same_state(pool, sim)
    # the safety arena runs dry in the middle of a batch: later requests report NOMEM, earlier ones moved
    rc, off, cap, st = pool.odma_migrate_batch([4, 5, 6], B.MIGRATE_DEFER_RELEASE)
    want = [sim.migrate(r, defer_release=True) for r in (4, 5, 6)]
    assert st.tolist() == [w[0] for w in want] and B.NOMEM in st.tolist() and rc == B.NOMEM
    # releasing a request whose source is still held frees both slabs
    assert pool.odma_release([4])[1].tolist() == sim.release([4])
    assert_same_state(pool, sim)
    pool.odma_release([r for r in range(22) if r != 4]); sim.release([r for r in range(22) if r != 4])
    assert_same_state(pool, sim)
    assert pool.odma_pool_free_extents(0) == [(0, 1 << 14)] and pool.odma_pool_free_extents(1) == [(1 << 14, 6 * 2048)]
