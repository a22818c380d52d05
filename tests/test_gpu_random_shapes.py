"""GPU parity on seeded random shapes: group size, KV heads, storage format, layout, launch shape and length mix are drawn
per case; every case goes through the C ABI and is compared with the oracle element by element (the bounds of the
format's own test module)."""
import math

import numpy as np
import pytest

import workloads as wl
from paper_2512_09427_amd import binding as B
from tests import harness as H
from tests.test_gpu_parity import TIGHT_F32, small_workload
from tests.test_gpu_fp8 import TIGHT_FP8

pytestmark = pytest.mark.gpu

FORMATS = [("bf16", 128), ("bf16", 64), ("fp8", 128), ("f32", 32), ("f32", 96), ("bf16", 32)]


def draw_lengths(rng, n):
    """A mix the method's workloads have: many short, a few block-aligned, a heavy tail; empties allowed."""
    kind = rng.integers(0, 4, n)
    short = rng.integers(0, 70, n)
    aligned = 16 * rng.integers(1, 40, n)
    mid = rng.integers(70, 1500, n)
    tail = np.minimum((128 * (1 - rng.random(n)) ** (-1 / 1.3)).astype(np.int64), 20000)
    return np.where(kind == 0, short, np.where(kind == 1, aligned, np.where(kind == 2, mid, tail))).astype(np.int64)


@pytest.mark.parametrize("seed", range(12))
def test_random_case(seed):
    rng = np.random.default_rng(9000 + seed)
    kv_dtype, d = FORMATS[seed % len(FORMATS)]
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    group = int(rng.integers(1, 17)) if d in (64, 128) and kv_dtype != "f32" else int(rng.integers(1, 9))
    n = int(rng.integers(1, 40))
    lens = draw_lengths(rng, n)
    paged = bool(rng.integers(0, 2))
    sharp = bool(rng.integers(0, 2))
    w = small_workload(lens, kv_dtype=kv_dtype, hq=hkv * group, hkv=hkv, d=d, seed=seed, bounds=(1024, 4096, 8192),
                       large_cap=20480, main=max(1, n) * 20480)
    dp = H.make_pool(w, out_dtype=B.F32)
    mfma = dp.pool.odma_pool_decode_kernel() == B.KERNEL_MFMA
    assert mfma == ((kv_dtype == "bf16" and d in (64, 128)) or kv_dtype == "fp8")
    if mfma:
        dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_CU, int(rng.choice([1, 4, 8, 16])))
        dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_WG, int(rng.choice([4, 8])))
        dp.pool.odma_pool_tune(B.TUNE_PIPELINE_DEPTH, int(rng.choice([2, 3])))
        dp.pool.odma_pool_tune(B.TUNE_FUSE_REDUCE, int(rng.integers(0, 2)))
    kv = [wl.request_kv(w, 0, r, sharp=sharp) for r in range(n)]
    q = wl.queries(w, 0, sharp=sharp)
    if paged:
        where = dict(block_table=wl.shuffled_block_table(lens, w.pool_tokens // 16, 16, seed=seed))
    else:
        where = dict(offsets=H.assign_perfect(dp, lens)[0])
    H.fill(dp, 0, kv, **where)
    got = H.decode(dp, 0, q, lens, **where)
    ref = H.oracle_out(w, q, kv, sm_scale=1.0 / math.sqrt(d))
    what = f"seed {seed}: {kv_dtype} d={d} hkv={hkv} G={group} n={n} paged={paged} sharp={sharp} max_len={int(lens.max())}"
    H.check(got, ref, what=what)
    a, r = TIGHT_FP8 if kv_dtype == "fp8" else (1e-5, 1e-5) if kv_dtype == "f32" else TIGHT_F32
    H.check(got, ref, a, r, what=what + " (tight)")
    assert (got[lens == 0] == 0).all()
    print(what)
