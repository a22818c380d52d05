"""Background recalibration thread of the library against the allocator oracle.

The set of boundaries that belongs to an epoch is a pure function of the completions reported
so far (the oracle computes it); which epoch an odma_assign call sees depends on timing, so the
library reports it and the oracle replays with exactly that set.  No GPU needed."""
import numpy as np
import pytest

import workloads as wl
from oracle import allocator as al
from paper_2512_09427_amd import binding as B
from tests.test_host_allocator import make_pair

BOUNDS = (512, 1024, 2048, 4096)


class EpochSets:
    """Boundaries per epoch from the oracle: completions folded in report order, `refresh` at a time."""

    def __init__(self, large_cap, window, refresh, bounds):
        self.cal = al.PoolSim(16, 16, large_cap, window=window, boundaries=bounds)
        self.refresh, self.pending, self.sets = refresh, [], [tuple(bounds)]

    def report(self, lengths):
        self.pending += [int(x) for x in lengths]

    def __getitem__(self, epoch):
        while len(self.sets) <= epoch:
            assert len(self.pending) >= self.refresh, "library published an epoch before its completions were reported"
            chunk, self.pending = self.pending[:self.refresh], self.pending[self.refresh:]
            self.sets.append(tuple(self.cal.recalibrate(chunk)))
        return self.sets[epoch]


def test_epochs_after_drain_are_deterministic():
    refresh, window = 50, 256
    pool, sim = make_pair(1 << 18, 4 * 65536, 65536, BOUNDS, max_requests=64, window=window)
    sets = EpochSets(65536, window, refresh, BOUNDS)
    rng = np.random.default_rng(11)
    pool.odma_recalibrator_start(refresh)
    total, rid = 0, 0
    for size in (1, 49, 50, 7, 243, 0, 100, 999):
        lens = wl.lognorm(rng, size, 700, 1.0, 1, 60000) if size else np.zeros(0, np.int64)
        pool.odma_report_completions(lens)
        sets.report(lens)
        total += size
        epoch = pool.odma_recalibrator_drain()
        assert epoch == total // refresh
        pred = [int(x) for x in wl.lognorm(rng, 3, 700, 1.0, 1, 60000)]
        ids = [rid, rid + 1, rid + 2]
        rid += 3
        rc, bk, off, cap, st = pool.odma_assign(ids, pred)
        stats = pool.odma_pool_stats()
        assert stats["boundary_epoch"] == epoch and stats["recalibrations"] == epoch
        assert pool.odma_pool_snapshot()[1] == sets[epoch]
        sim.boundaries = sets[epoch]
        assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(map(list, sim.assign(ids, pred)))
    pool.odma_recalibrator_stop()
    assert pool.odma_pool_snapshot()[1] == sets[total // refresh]
    # the window now belongs to the caller again, in the state the thread left it
    more = [int(x) for x in wl.lognorm(rng, 10, 300, 0.5, 1, 60000)]
    sets.cal.boundaries = sets[total // refresh]
    assert pool.odma_recalibrate(more) == tuple(sets.cal.recalibrate(sets.pending + more))


def test_free_running_thread_replays_bit_exactly():
    """Config 5's host loop with completions reported to the thread and no synchronisation with it."""
    slots, steps, refresh, window = 48, 400, 25, 256
    pool, sim = make_pair(1 << 18, 4 * 65536, 65536, BOUNDS, max_requests=slots, window=window)
    sets = EpochSets(65536, window, refresh, BOUNDS)
    pool.odma_recalibrator_start(refresh)
    gen = wl.drift_arrivals(seed=5, n_steps=steps)
    next(gen)
    live, reported, epochs = {}, 0, []
    for step in range(steps):
        for s in range(slots):
            if s in live:
                continue
            a = gen.send(step)
            rc, bk, off, cap, st = pool.odma_assign([s], [a.pred_len], np.array([a.uncertainty], np.float32))
            epoch = pool.odma_pool_stats()["boundary_epoch"]
            epochs.append(epoch)
            sim.boundaries = sets[epoch]
            want = sim.assign([s], [a.pred_len], [np.float32(a.uncertainty)])
            assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(map(list, want))
            if st[0] != 0:
                continue
            ov = pool.odma_advance([s], [a.prefilled])[1]
            assert ov.tolist() == sim.advance([s], [a.prefilled])[0]
            if ov[0]:
                assert pool.odma_migrate(s)[:2] == sim.migrate(s)[:2]
                assert pool.odma_advance([s], [a.prefilled])[1].tolist() == sim.advance([s], [a.prefilled])[0]
            live[s] = [a.total_len, a.prefilled]
        ids = sorted(live)
        ov = pool.odma_advance(ids)[1]
        assert ov.tolist() == sim.advance(ids)[0]
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
            lens = [live[s][0] for s in fin]
            assert pool.odma_release(fin)[1].tolist() == sim.release(fin)
            pool.odma_report_completions(lens)
            sets.report(lens)
            reported += len(lens)
            for s in fin:
                del live[s]
    assert epochs == sorted(epochs)
    pool.odma_recalibrator_stop()
    final = reported // refresh
    assert final >= 10 and pool.odma_pool_stats()["boundary_epoch"] == final
    rows, bounds = pool.odma_pool_snapshot()
    assert bounds == sets[final] and rows == [tuple(r) for r in sim.snapshot()]
    for arena in (0, 1):
        assert pool.odma_pool_free_extents(arena) == sim.free_extents(arena)


def test_recalibrator_call_order_errors():
    pool, _ = make_pair(1 << 12, 1 << 12, 1 << 12, (64, 128, 256), max_requests=8)
    for call in (lambda: pool.odma_report_completions([5]), pool.odma_recalibrator_drain, pool.odma_recalibrator_stop):
        with pytest.raises(B.OdmaError):
            call()
    with pytest.raises(B.OdmaError):
        pool.odma_recalibrator_start(0)
    pool.odma_recalibrator_start(2)
    with pytest.raises(B.OdmaError):
        pool.odma_recalibrator_start(2)
    with pytest.raises(B.OdmaError):
        pool.odma_recalibrate([5])                 # the thread owns the window
    pool.odma_report_completions([100, 100, 100])
    assert pool.odma_recalibrator_drain() == 1
    pool.close()                                   # destroying the pool stops the thread
    two, _ = make_pair(1 << 12, 1 << 12, 1 << 12, (64, 128), max_requests=8)     # B = 2: no default quantile levels
    with pytest.raises(B.OdmaError):
        two.odma_recalibrator_start(10)
