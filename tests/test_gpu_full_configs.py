"""Configurations 4 and 5 at their stated size and protocol, and the in-kernel merge under many launches.

Configuration 4 (28 layers, batch 128, the seeded overflows migrating in mid-run) runs the path ``bench.py`` times:
``odma_advance`` -> ``odma_migrate_batch`` -> 28 x fused ``odma_decode_step`` with ``ODMA_REUSE_PLAN`` from the second
layer on, with fewer steps than the bench so that the attention oracle can look at three layers in every step.
Configuration 5 runs its full 1 000 steps.  The drivers are in ``tests/scenarios.py``.
"""
import numpy as np
import pytest

import workloads as wl
from paper_2512_09427_amd import binding as B
from tests import harness as H
from tests import scenarios as S
from tests.test_gpu_parity import TIGHT_F32, small_workload

pytestmark = pytest.mark.gpu


def test_config4_28_layers_fused_steps_with_batched_migration():
    res = S.run_config4(steps=10, n_layers=28, check_layers=(0, 13, 27), check_steps=None)
    assert res["layers"] == 28 and res["requests"] == 128 and res["migrations"] == 6
    assert res["oracle_checked_steps"] == 10 and res["check_layers"] == [0, 13, 27]
    assert len(res["migration_copies"]) >= 1 and sum(m["requests"] for m in res["migration_copies"]) == 6
    print(f"config 4: {res['ms_per_step_median']:.3f} ms/step over 28 layers, {res['kv_GBps']:.0f} GB/s, "
          f"max err / max|ref| {res['max_err_over_max_ref']:.2e}")


def test_config5_full_drift_run():
    res = S.run_config5(steps=1000, slots=256, clip=65536, window=2048, recal_every=100, check_every=100)
    assert res["recalibrations"] == 10 and len(res["boundary_trajectory"]) == 11
    assert res["completed"] > 3000 and res["oracle_checked_steps"] >= 10 and res["oracle_checked_requests"] >= 40
    assert 0.0 < res["utilization_completed"] <= 1.0 and res["sustained_kv_GBps"] > 100
    sets = [tuple(t["boundaries"]) for t in res["boundary_trajectory"]]
    assert all(all(x < y for x, y in zip(b, b[1:])) and all(x % 16 == 0 for x in b) for b in sets)
    assert len(set(sets)) >= 5                                         # the boundaries follow the drifting lengths
    assert res["admitted"] >= res["completed"]
    print(f"config 5: {res['completed']} completed, utilization {res['utilization_completed']:.3f}, "
          f"{res['migrations']} migrations, {res['nomem']} NOMEM, {res['sustained_kv_GBps']:.0f} GB/s, boundaries {sets}")


def test_in_kernel_merge_over_two_hundred_launches():
    """The merge of cut segments inside the attention launch (arrival counters, partial states crossing between
    work-groups) against the separate reduction launch and the oracle: 200 launches over seeded random length sets
    with cuts of two up to tens of parts, empty requests, the plan reused and not, stopping at the first mismatch.
    The two merges add the parts in different batch sizes, so they agree to rounding (1e-6 relative), not bit for bit."""
    rng = np.random.default_rng(2024)
    launches = 0
    for case in range(25):
        n = int(rng.integers(3, 40))
        kind = case % 5
        if kind == 0:                                                  # one very long request among short ones
            lens = rng.integers(0, 300, n)
            lens[rng.integers(n)] = int(rng.integers(20000, 60000))
        elif kind == 1:                                                # several long requests: cuts of 5..20 parts
            lens = rng.integers(2000, 12000, n)
        elif kind == 2:                                                # many short ones: two-part cuts everywhere
            lens = rng.integers(1, 700, n)
        elif kind == 3:                                                # few tiles: fewer waves used than launched
            lens = rng.integers(0, 40, n)
        else:                                                          # heavy tail
            lens = np.minimum(wl.pareto(rng, n, 1.2, 64, 40000), 40000)
        lens = np.asarray(lens, dtype=np.int64)
        lens[rng.integers(n)] = 0
        w = small_workload(lens, seed=300 + case, bounds=(1024, 8192, 65536), large_cap=65536,
                           main=int(((np.maximum(lens, 1) + 65535) // 65536 * 65536).sum()), safety=65536)
        dp = H.make_pool(w, out_dtype=B.F32)
        off, _ = H.assign_perfect(dp, np.maximum(lens, 1))
        kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
        q = wl.queries(w, 0, sharp=True)
        H.fill(dp, 0, kv, offsets=off)
        ref = H.oracle_out(w, q, kv)
        ref[lens == 0] = 0.0
        dp.pool.odma_pool_tune(B.TUNE_FUSE_REDUCE, 0)
        separate = H.decode(dp, 0, q, lens, offsets=off)
        H.check(separate, ref, *TIGHT_F32, what=f"case {case}: reduction launch")
        dp.pool.odma_pool_tune(B.TUNE_FUSE_REDUCE, 1)
        for launch in range(8):
            flags = B.REUSE_PLAN if launch % 2 else 0
            got = H.decode(dp, 0, q, lens, offsets=off, flags=flags)
            launches += 1
            what = f"case {case} (kind {kind}, {n} requests, longest {int(lens.max())}), launch {launch}, flags {flags}"
            H.check(got, ref, *TIGHT_F32, what=what)
            np.testing.assert_allclose(got, separate, rtol=1e-6, atol=1e-7, err_msg=what)
    assert launches == 200
