"""GPU parity: libodma through its C ABI against the CPU oracle, element by element.

Tolerance (stated by the benchmark spec for bf16-in / fp32-accumulate attention):
|gpu - oracle| <= 2e-3 + 1e-2 * |oracle|.  Because the seeded configurations scale their
data by 1/sqrt(128), |out| is only a few 1e-3 there and the absolute term alone would
hide mistakes; every case therefore also runs a "sharp" variant (unscaled Q and K, peaked
softmax) and asserts the much tighter engineering bound the kernels are built to
(fp32 output: 2e-5 + 2e-4*|ref|; bf16 output: one bf16 rounding on top of that).
Offsets, assignments and migrations are compared bit-exactly.
"""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import allocator as al
from oracle import attention as oa
from paper_2512_09427_amd import binding as B
from tests import harness as H

pytestmark = pytest.mark.gpu

TIGHT_F32 = (2e-5, 2e-4)
TIGHT_BF16 = (2e-5, 2e-4 + 2.0 ** -8)


def tight(out_dtype):
    return TIGHT_BF16 if out_dtype == B.BF16 else TIGHT_F32


def small_workload(lengths, kv_dtype="bf16", hq=28, hkv=4, d=128, seed=0, bounds=(1024, 2048, 4096), large_cap=4096,
                   main=None, safety=None):
    lengths = np.asarray(lengths, dtype=np.int64)
    main = main if main is not None else max(1, len(lengths)) * large_cap
    return wl.Workload("case", 1, hq, hkv, d, kv_dtype, lengths, bounds, main_tokens=main,
                       safety_tokens=safety if safety is not None else 4 * large_cap, large_cap=large_cap,
                       data_seed=1000 + seed, data_scale=1.0 / math.sqrt(d))


def pin_launch_shape(dp, waves_per_cu=4, waves_per_wg=4):
    """Results are bit-identical across layouts for one launch shape (the split of the tile stream fixes the
    summation order): the comparisons pin it rather than rely on the defaults being equal."""
    dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_CU, waves_per_cu)
    dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_WG, waves_per_wg)


def run_case(w, *, kernel=B.KERNEL_AUTO, out_dtype=None, sharp=False, paged=False, tol=None, max_splits=0, pin=False):
    dp = H.make_pool(w, decode_kernel=kernel, out_dtype=out_dtype, max_splits=max_splits)
    if pin:
        pin_launch_shape(dp)
    n = w.n_requests
    kv = [wl.request_kv(w, 0, r, sharp=sharp) for r in range(n)]
    q = wl.queries(w, 0, sharp=sharp)
    if paged:
        bt = wl.shuffled_block_table(w.lengths, w.pool_tokens // 16, 16, seed=77)
        H.fill(dp, 0, kv, block_table=bt)
        got = H.decode(dp, 0, q, w.lengths, block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, w.lengths)
        H.fill(dp, 0, kv, offsets=off)
        got = H.decode(dp, 0, q, w.lengths, offsets=off)
    ref = H.oracle_out(w, q, kv)
    H.check(got, ref, what=w.name)                                   # the stated tolerance
    a, r = tol if tol is not None else tight(dp.out_dtype)
    return H.check(got, ref, a, r, what=w.name + " (tight)"), got, dp


# ---- config 1: Tiny, fp32 ----------------------------------------------------------------------

@pytest.mark.parametrize("paged", [False, True])
def test_tiny_fp32(paged):
    w = wl.tiny()
    rel, got, dp = run_case(w, paged=paged, tol=(1e-5, 1e-5))
    assert dp.pool.odma_pool_decode_kernel() == B.KERNEL_VALU
    # oracle in its fp32 mode agrees too (the plain fp32 CPU implementation)
    kv = [wl.request_kv(w, 0, r) for r in range(4)]
    H.check(got, H.oracle_out(w, wl.queries(w, 0), kv, np.float32).astype(np.float64), 1e-5, 1e-5)


def test_tiny_assignment_and_migration_are_bit_exact_and_migration_preserves_output():
    w = wl.tiny()
    dp = H.make_pool(w)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries)
    pred = [60] + w.lengths.tolist()[1:]
    rc, bk, off, cap, st = dp.pool.odma_assign(range(4), pred)
    assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(sim.assign(range(4), pred))
    kv = [wl.request_kv(w, 0, r) for r in range(4)]
    first = [(k[:64], v[:64]) if r == 0 else (k, v) for r, (k, v) in enumerate(kv)]
    H.fill(dp, 0, first, offsets=off)
    lens = np.array([64, 73, 101, 123])
    dp.pool.odma_advance(range(4), lens); sim.advance(range(4), lens.tolist())
    q = wl.queries(w, 0)
    before = H.decode(dp, 0, q, lens, offsets=off)
    assert dp.pool.odma_advance([0])[1].tolist() == sim.advance([0])[0] == [1]
    rc, noff, ncap = dp.pool.odma_migrate(0)
    assert (rc, noff, ncap) == sim.migrate(0)[:3] == (0, 1024, 256)
    off2 = off.copy(); off2[0] = noff
    after = H.decode(dp, 0, q, lens, offsets=off2)
    np.testing.assert_array_equal(before, after)                      # same kernel, same chunking
    gk, gv = H.gather(dp, 0, noff, 64)
    np.testing.assert_array_equal(gk, kv[0][0][:64]); np.testing.assert_array_equal(gv, kv[0][1][:64])
    # the remaining tokens land in the Large-Bucket slab and the full result matches the oracle
    H.fill(dp, 0, [(kv[0][0][64:], kv[0][1][64:])], offsets=np.array([noff]), positions=np.array([64]))
    got = H.decode(dp, 0, q, w.lengths, offsets=off2)
    H.check(got, H.oracle_out(w, q, kv), 1e-5, 1e-5, "tiny after migration")
    assert dp.pool.odma_pool_snapshot()[0] == [tuple(r) for r in sim.snapshot()]


# ---- config 2: Qwen2-7B shape, batch 64 -----------------------------------------------------------

@pytest.mark.parametrize("kernel", [B.KERNEL_MFMA, B.KERNEL_VALU])
@pytest.mark.parametrize("out_dtype", [B.BF16, B.F32])
@pytest.mark.parametrize("sharp", [False, True])
def test_config2_contiguous(kernel, out_dtype, sharp):
    rel, _, dp = run_case(wl.qwen_b64(), kernel=kernel, out_dtype=out_dtype, sharp=sharp)
    assert dp.pool.odma_pool_decode_kernel() == kernel
    print(f"config2 kernel={kernel} out={out_dtype} sharp={sharp}: max err / max|ref| = {rel:.2e}")


@pytest.mark.parametrize("kernel", [B.KERNEL_MFMA, B.KERNEL_VALU])
def test_config2_paged_equals_contiguous_bitwise(kernel):
    w = wl.qwen_b64()
    _, got_c, _ = run_case(w, kernel=kernel, out_dtype=B.F32, sharp=True, pin=True)
    _, got_p, _ = run_case(w, kernel=kernel, out_dtype=B.F32, sharp=True, paged=True, pin=True)
    np.testing.assert_array_equal(got_c, got_p)                        # layout must not change a single bit
    run_case(w, kernel=kernel, out_dtype=B.F32, sharp=True, paged=True)   # and the paged layout's own launch shape


# ---- edge cases ------------------------------------------------------------------------------------

@pytest.mark.parametrize("kernel", [B.KERNEL_MFMA, B.KERNEL_VALU])
def test_ragged_and_degenerate_lengths(kernel):
    lens = [0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 63, 64, 65, 127, 128, 129, 255, 256, 257, 0, 1000, 1024, 4096, 3]
    w = small_workload(lens, seed=1)
    for sharp in (False, True):
        rel, got, _ = run_case(w, kernel=kernel, out_dtype=B.F32, sharp=sharp)
        assert (got[0] == 0).all() and (got[19] == 0).all()            # empty requests give zeros
        # len == 1: the output is that value row exactly (softmax weight 1, bf16 values exact in fp32)
        k, v = wl.request_kv(w, 0, 1, sharp=sharp)
        for h in range(28):
            np.testing.assert_array_equal(got[1, h], wl.bf16_bits_to_f32(v[0, h // 7]))


def test_single_request_and_other_group_sizes():
    for (hq, hkv, d, kvd) in [(4, 4, 128, "bf16"), (16, 1, 128, "bf16"), (8, 2, 64, "bf16"), (6, 2, 32, "f32"),
                              (3, 1, 256, "f32"), (32, 2, 128, "bf16")]:
        w = small_workload([333], kv_dtype=kvd, hq=hq, hkv=hkv, d=d, seed=hq)
        rel, _, dp = run_case(w, out_dtype=B.F32, sharp=True)
        want = B.KERNEL_MFMA if (kvd == "bf16" and d in (64, 128)) else B.KERNEL_VALU
        assert dp.pool.odma_pool_decode_kernel() == want


def test_every_launch_shape_gives_the_same_answer():
    """Launch-shape knobs change who computes what, never the result: waves per CU, work-group size, register
    buffers, weights, in-kernel merge, each with the contiguous, the paged and the fused path."""
    lens = np.array([2100, 17, 0, 640, 16, 9000, 1, 333, 48, 1279, 15, 4096], dtype=np.int64)
    w = small_workload(lens, seed=31, bounds=(1024, 4096, 16384), large_cap=16384)
    n = len(lens)
    kv = [wl.request_kv(w, 0, r, n_tokens=int(lens[r]) + 1, sharp=True) for r in range(n)]
    held = [(k[:lens[r]], v[:lens[r]]) for r, (k, v) in enumerate(kv)]
    q = wl.queries(w, 0, sharp=True)
    ref = H.oracle_out(w, q, held)
    ref_next = H.oracle_out(w, q, kv)                                  # after one more token per request
    for r in range(n):
        if lens[r] == 0:
            ref[r] = 0.0
    k_new = np.stack([kv[r][0][lens[r]] for r in range(n)])
    v_new = np.stack([kv[r][1][lens[r]] for r in range(n)])
    bt = wl.shuffled_block_table(lens + 1, w.pool_tokens // 16, 16, seed=32)
    shapes = [dict(), dict(cu=8, wg=8), dict(cu=8, wg=4), dict(cu=4, wg=4, depth=3), dict(cu=8, wg=8, depth=3),
              dict(cu=16, wg=8), dict(cu=1, wg=4), dict(cu=4, wg=4, odd=200, late=300), dict(cu=8, wg=8, fuse=1),
              dict(cu=4, wg=4, fuse=1, depth=3)]
    for paged in (False, True):
        for shape in shapes:
            dp = H.make_pool(w, out_dtype=B.F32)
            for knob, key in ((B.TUNE_WAVES_PER_CU, "cu"), (B.TUNE_WAVES_PER_WG, "wg"), (B.TUNE_PIPELINE_DEPTH, "depth"),
                              (B.TUNE_ODD_XCD_WEIGHT, "odd"), (B.TUNE_LATE_WAVE_WEIGHT, "late"), (B.TUNE_FUSE_REDUCE, "fuse")):
                if key in shape:
                    dp.pool.odma_pool_tune(knob, shape[key])
            if paged:
                off = None
                H.fill(dp, 0, held, block_table=bt)
            else:
                off, _ = H.assign_perfect(dp, lens + 1)
                H.fill(dp, 0, held, offsets=off)
            what = f"paged={paged} {shape}"
            got = H.decode(dp, 0, q, lens, offsets=off, block_table=bt if paged else None)
            H.check(got, ref, *TIGHT_F32, what=what)
            got = H.decode_step(dp, 0, q, k_new, v_new, lens + 1, offsets=off, block_table=bt if paged else None)
            H.check(got, ref_next, *TIGHT_F32, what=what + " fused step")
            again = H.decode(dp, 0, q, lens + 1, offsets=off, block_table=bt if paged else None)
            np.testing.assert_array_equal(got, again)                  # the appended rows are in the pool


def test_thousands_of_short_requests():
    """More requests than plan threads and than one 64-entry window: entries, windows and ranges all roll over."""
    rng = np.random.default_rng(41)
    lens = rng.integers(0, 40, 3000).astype(np.int64)
    lens[rng.integers(0, 3000, 20)] = 0
    w = small_workload(lens, seed=41, bounds=(64, 128, 256), large_cap=256, main=3000 * 64, safety=1024)
    rel, got, _ = run_case(w, out_dtype=B.F32, sharp=True)
    assert (got[lens == 0] == 0).all()
    run_case(w, out_dtype=B.BF16, sharp=False, paged=True)


@pytest.mark.parametrize("kernel", [B.KERNEL_MFMA, B.KERNEL_VALU])
def test_long_requests_split_over_many_chunks(kernel):
    # one 32768-token request next to short ones: the heavy-tail case of config 3
    w = small_workload([32768, 129, 5000, 64], seed=2, bounds=(1024, 8192, 32768), large_cap=32768)
    run_case(w, kernel=kernel, out_dtype=B.F32, sharp=True)
    run_case(w, kernel=kernel, out_dtype=B.BF16, sharp=False)
    # a tiny work-list budget forces large chunks; results must still match
    run_case(w, kernel=kernel, out_dtype=B.F32, sharp=True, max_splits=3)


@pytest.mark.parametrize("out_dtype", [B.F32, B.BF16])
def test_in_kernel_merge_of_cut_segments(out_dtype):
    """ODMA_TUNE_FUSE_REDUCE = 1: the last work-group to finish a segment cut by work-group boundaries merges
    it inside the attention launch.  Same answer as the separate reduction launch, on repeated launches (the
    arrival counters must return to zero), for chains of 2 and of tens of work-groups, and for empty requests."""
    lengths = [32768, 0, 129, 5000, 64, 0, 9000, 1, 700]
    w = small_workload(lengths, seed=12, bounds=(1024, 8192, 32768), large_cap=32768)
    dp = H.make_pool(w, out_dtype=out_dtype)
    off, _ = H.assign_perfect(dp, np.maximum(w.lengths, 1))
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(w.n_requests)]
    q = wl.queries(w, 0, sharp=True)
    H.fill(dp, 0, kv, offsets=off)
    ref = H.oracle_out(w, q, kv)
    for r, n_tok in enumerate(lengths):
        if n_tok == 0:
            ref[r] = 0.0
    separate = H.decode(dp, 0, q, w.lengths, offsets=off)
    H.check(separate, ref, *tight(out_dtype), what="separate reduction")
    dp.pool.odma_pool_tune(B.TUNE_FUSE_REDUCE, 1)
    for launch in range(3):
        fused = H.decode(dp, 0, q, w.lengths, offsets=off, flags=B.REUSE_PLAN if launch == 2 else 0)
        H.check(fused, ref, *tight(out_dtype), what=f"in-kernel merge, launch {launch}")
        np.testing.assert_allclose(fused, separate, rtol=2e-2 if out_dtype == B.BF16 else 1e-5, atol=1e-6)


def test_dominant_key_far_from_first_tile():
    """Running-max update: a late token dominates, earlier accumulators must be rescaled away."""
    w = small_workload([700], seed=3)
    dp = H.make_pool(w, out_dtype=B.F32)
    off, _ = H.assign_perfect(dp, w.lengths)
    k, v = wl.request_kv(w, 0, 0, sharp=True)
    q = wl.queries(w, 0, sharp=True)
    qf = wl.bf16_bits_to_f32(q[0])
    for g in range(4):                                                 # token 650 aligns with head 7g's query
        k[650, g] = wl.f32_to_bf16_bits(4.0 * qf[7 * g])
    H.fill(dp, 0, [(k, v)], offsets=off)
    got = H.decode(dp, 0, q, w.lengths, offsets=off)
    ref = H.oracle_out(w, q, [(k, v)])
    H.check(got, ref, *TIGHT_F32, what="dominant key")
    np.testing.assert_allclose(got[0, 0], wl.bf16_bits_to_f32(v[650, 0]), atol=1e-6)


# ---- append path ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("paged", [False, True])
def test_stepwise_append_then_attention(paged):
    """Config-4 order: each step appends one token per request, then attends over len+1 tokens."""
    lens0 = np.array([5, 14, 15, 16, 31, 200], dtype=np.int64)
    steps = 20
    w = small_workload(lens0, seed=4)
    dp = H.make_pool(w, out_dtype=B.F32)
    n = len(lens0)
    kv = [list(wl.request_kv(w, 0, r, n_tokens=int(lens0[r]) + steps, sharp=True)) for r in range(n)]
    bt = off = None
    if paged:
        bt = wl.shuffled_block_table(lens0 + steps, w.pool_tokens // 16, 16, seed=5)
        H.fill(dp, 0, [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)], block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, lens0, extra=steps)
        H.fill(dp, 0, [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)], offsets=off)
    lens = lens0.copy()
    for s in range(steps):
        k_new = np.stack([kv[r][0][lens[r]] for r in range(n)])
        v_new = np.stack([kv[r][1][lens[r]] for r in range(n)])
        H.append_one(dp, 0, k_new, v_new, lens, offsets=off, block_table=bt)
        lens += 1
        q = wl.queries(w, 0, step=s, sharp=True)
        got = H.decode(dp, 0, q, lens, offsets=off, block_table=bt)
        ref = H.oracle_out(w, q, [(kv[r][0][:lens[r]], kv[r][1][:lens[r]]) for r in range(n)])
        H.check(got, ref, *TIGHT_F32, what=f"step {s}")


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("shape", [("bf16", 28, 4, 128), ("f32", 4, 2, 64)])
def test_fused_decode_step_equals_append_then_attention(paged, shape):
    """odma_decode_step: same outputs as the oracle on len+1 tokens, and the appended rows are in the
    pool afterwards (read back through odma_gather_kv), across block boundaries and split requests."""
    kvd, hq, hkv, d = shape
    lens0 = np.array([0, 1, 14, 15, 16, 17, 31, 32, 200, 3000, 555], dtype=np.int64)
    steps = 18
    w = small_workload(lens0, kv_dtype=kvd, hq=hq, hkv=hkv, d=d, seed=11)
    dp = H.make_pool(w, out_dtype=B.F32)
    n = len(lens0)
    kv = [list(wl.request_kv(w, 0, r, n_tokens=int(lens0[r]) + steps, sharp=True)) for r in range(n)]
    bt = off = None
    if paged:
        bt = wl.shuffled_block_table(lens0 + steps, w.pool_tokens // 16, 16, seed=12)
        H.fill(dp, 0, [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)], block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, lens0, extra=steps)
        H.fill(dp, 0, [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)], offsets=off)
    lens = lens0.copy()
    tol = TIGHT_F32 if kvd == "bf16" else (1e-5, 1e-5)
    for s in range(steps):
        k_new = np.stack([kv[r][0][lens[r]] for r in range(n)])
        v_new = np.stack([kv[r][1][lens[r]] for r in range(n)])
        lens += 1
        q = wl.queries(w, 0, step=s, sharp=True)
        got = H.decode_step(dp, 0, q, k_new, v_new, lens, offsets=off, block_table=bt)
        ref = H.oracle_out(w, q, [(kv[r][0][:lens[r]], kv[r][1][:lens[r]]) for r in range(n)])
        H.check(got, ref, *tol, what=f"fused step {s}")
    for r in (1, 4, 9):
        gk, gv = H.gather(dp, 0, 0 if paged else int(off[r]), int(lens[r]), block_row=bt[r] if paged else None)
        np.testing.assert_array_equal(gk, kv[r][0][:lens[r]]); np.testing.assert_array_equal(gv, kv[r][1][:lens[r]])


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 128), ("f32", 64)])
def test_append_gather_round_trip_is_bit_exact(kv_dtype, d):
    lens = [1, 16, 17, 250]
    w = small_workload(lens, kv_dtype=kv_dtype, hq=4, hkv=2, d=d, seed=6)
    dp = H.make_pool(w)
    kv = [wl.request_kv(w, 0, r) for r in range(4)]
    off, _ = H.assign_perfect(dp, w.lengths)
    H.fill(dp, 0, kv, offsets=off)
    for r in range(4):
        gk, gv = H.gather(dp, 0, int(off[r]), lens[r])
        np.testing.assert_array_equal(gk, kv[r][0]); np.testing.assert_array_equal(gv, kv[r][1])
    # paged: same rows through a shuffled block table
    dp2 = H.make_pool(w)
    bt = wl.shuffled_block_table(w.lengths, w.pool_tokens // 16, 16, seed=8)
    H.fill(dp2, 0, kv, block_table=bt)
    for r in range(4):
        gk, gv = H.gather(dp2, 0, 0, lens[r], block_row=bt[r])
        np.testing.assert_array_equal(gk, kv[r][0]); np.testing.assert_array_equal(gv, kv[r][1])


# ---- config 3: batch 256, Pareto lengths, contiguous vs paged on identical data ---------------------------

def test_config3_full_size_contiguous_and_paged():
    w = wl.qwen_b256_pareto()
    n = w.n_requests
    kv = [wl.request_kv(w, 0, r) for r in range(n)]
    q = wl.queries(w, 0)
    ref = H.oracle_out(w, q, kv)
    # contiguous: boundaries recalibrated on the batch itself, as the configuration says
    dp = H.make_pool(w, out_dtype=B.F32)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries, max_requests=n)
    assert dp.pool.odma_recalibrate(w.lengths.tolist()) == tuple(sim.recalibrate(w.lengths.tolist()))
    rc, bk, off, cap, st = dp.pool.odma_assign(range(n), w.lengths)
    assert rc == 0
    assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(sim.assign(range(n), w.lengths.tolist()))
    H.fill(dp, 0, kv, offsets=off)
    got_c = H.decode(dp, 0, q, w.lengths, offsets=off)
    rel = H.check(got_c, ref, what="config3 contiguous")
    H.check(got_c, ref, *TIGHT_F32, what="config3 contiguous (tight)")
    # paged: same logical K/V in a shuffled 16-token-block pool
    dp2 = H.make_pool(w, out_dtype=B.F32)
    bt = wl.shuffled_block_table(w.lengths, w.pool_tokens // 16, 16, seed=w.extra["page_seed"], max_blocks=2048)
    H.fill(dp2, 0, kv, block_table=bt)
    got_p = H.decode(dp2, 0, q, w.lengths, block_table=bt)            # the paged layout's own launch shape
    H.check(got_p, ref, *TIGHT_F32, what="config3 paged (tight)")
    pin_launch_shape(dp2)                                             # the contiguous one: not a bit may differ
    got_p = H.decode(dp2, 0, q, w.lengths, block_table=bt)
    np.testing.assert_array_equal(got_c, got_p)
    print(f"config3: max err / max|ref| = {rel:.2e}")


# ---- config 4: multi-layer decode steps with overflow -> migration ------------------------------------------

def test_config4_decode_steps_with_migration():
    """28-layer shape reduced to 2 layers and 12 steps so the CPU oracle stays fast; batch 128,
    the seeded 5 % overflow set migrates mid-run.  Host decisions are compared with the allocator
    oracle bit for bit, attention with the attention oracle at every step on layer 0 and 1."""
    steps, L = 8, 2
    w = wl.qwen_b128_step(n_layers=L, steps=steps)
    n = w.n_requests
    dp = H.make_pool(w, out_dtype=B.BF16)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries, max_requests=n)
    lens = w.lengths.copy()
    pred = (lens + steps).copy()
    # overflowing requests: slab = bucket of len0, start at cap - k so that step k+1 overflows
    caps0 = np.array([min(b for b in w.boundaries if b >= x) for x in lens])
    for r, kk in zip(w.extra["overflow_req"], np.minimum(w.extra["overflow_after"], steps - 2)):
        pred[r] = caps0[r]
        lens[r] = caps0[r] - kk
    rc, bk, off, cap, st = dp.pool.odma_assign(range(n), pred)
    assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(sim.assign(range(n), pred.tolist()))
    total = lens + steps
    kv = [[wl.request_kv(w, l, r, n_tokens=int(total[r])) for r in range(n)] for l in range(L)]
    for l in range(L):
        H.fill(dp, l, [(k[:lens[r]], v[:lens[r]]) for r, (k, v) in enumerate(kv[l])], offsets=off)
    dp.pool.odma_advance(range(n), lens); sim.advance(range(n), lens.tolist())
    migrated = 0
    off = off.copy()
    for s in range(steps):
        rc, ov, _ = dp.pool.odma_advance(range(n)); sov, _ = sim.advance(range(n))
        assert ov.tolist() == sov
        for r in np.nonzero(ov)[0]:
            got, want = dp.pool.odma_migrate(int(r)), sim.migrate(int(r))
            assert got == want[:3] and got[0] == 0
            off[r] = got[1]
            migrated += 1
            assert dp.pool.odma_advance([int(r)])[1].tolist() == sim.advance([int(r)])[0] == [0]
        for l in range(L):
            k_new = np.stack([kv[l][r][0][lens[r]] for r in range(n)])
            v_new = np.stack([kv[l][r][1][lens[r]] for r in range(n)])
            H.append_one(dp, l, k_new, v_new, lens, offsets=off)
            q = wl.queries(w, l, step=s)
            got = H.decode(dp, l, q, lens + 1, offsets=off, flags=B.REUSE_PLAN if l > 0 else 0)
            ref = H.oracle_out(w, q, [(kv[l][r][0][:lens[r] + 1], kv[l][r][1][:lens[r] + 1]) for r in range(n)])
            H.check(got, ref, what=f"config4 step {s} layer {l}")
            H.check(got, ref, *TIGHT_BF16, what=f"config4 step {s} layer {l} (tight)")
        lens += 1
        assert dp.pool.odma_pool_lookup(range(n))[1].tolist() == lens.tolist()
    assert migrated == len(w.extra["overflow_req"]) == sim.n_migrations
    assert dp.pool.odma_pool_snapshot()[0] == [tuple(r) for r in sim.snapshot()]


def test_batched_migration_on_a_side_stream():
    """odma_migrate_batch with deferred release: the copies run on a stream of their own while the other requests
    decode; afterwards the migrated requests read bit-identical K/V from their Large-Bucket slabs."""
    import torch
    lens = np.array([700, 64, 1500, 33, 900, 260, 15, 1200], dtype=np.int64)
    w = small_workload(lens, seed=21, bounds=(1024, 2048, 4096), large_cap=4096, safety=8 * 4096)
    dp = H.make_pool(w, out_dtype=B.F32, n_layers=1)
    off, _ = H.assign_perfect(dp, lens)
    dp.pool.odma_advance(range(len(lens)), lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(len(lens))]
    q = wl.queries(w, 0, sharp=True)
    H.fill(dp, 0, kv, offsets=off)
    before = H.decode(dp, 0, q, lens, offsets=off)
    movers, others = [0, 2, 5], [1, 3, 4, 6, 7]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    rc, noff, ncap, st = dp.pool.odma_migrate_batch(movers, B.MIGRATE_DEFER_RELEASE, stream=side)
    assert rc == 0 and st.tolist() == [0, 0, 0] and ncap.tolist() == [4096] * 3
    assert all(o >= w.main_tokens for o in noff)
    # the others keep decoding on the compute stream; an admission now cannot be handed a source slab
    got = H.decode(dp, 0, q[others], lens[others], offsets=off[others])
    H.check(got, H.oracle_out(w, q[others], [kv[r] for r in others]), *TIGHT_F32, what="others during the copy")
    new_off = dp.pool.odma_assign([8], [64])[2][0]
    assert all(not (off[m] <= new_off < off[m] + 64) for m in movers)
    torch.cuda.current_stream().wait_stream(side)
    assert dp.pool.odma_migrate_finish(movers)[1].tolist() == [0, 0, 0]
    off2 = off.copy()
    off2[movers] = noff
    after = H.decode(dp, 0, q, lens, offsets=off2)
    np.testing.assert_array_equal(before, after)
    for m in movers:
        gk, gv = H.gather(dp, 0, int(off2[m]), int(lens[m]))
        np.testing.assert_array_equal(gk, kv[m][0]); np.testing.assert_array_equal(gv, kv[m][1])
    # without the flag a batch is the sequence of single migrations
    rc, noff2, _, st2 = dp.pool.odma_migrate_batch([4, 7])
    assert rc == 0 and st2.tolist() == [0, 0]
    off2[[4, 7]] = noff2
    np.testing.assert_array_equal(before, H.decode(dp, 0, q, lens, offsets=off2))


def test_reuse_plan_flag_gives_identical_results():
    w = small_workload([700, 3000, 40], seed=9)
    dp = H.make_pool(w, out_dtype=B.F32)
    off, _ = H.assign_perfect(dp, w.lengths)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(3)]
    H.fill(dp, 0, kv, offsets=off)
    q = wl.queries(w, 0, sharp=True)
    a = H.decode(dp, 0, q, w.lengths, offsets=off)
    b = H.decode(dp, 0, q, w.lengths, offsets=off, flags=B.REUSE_PLAN)
    np.testing.assert_array_equal(a, b)


def test_reuse_plan_after_migration_and_after_a_layout_switch():
    """A matrix-core plan bakes the slab bases in.  After a migration (offsets change, lengths do not) or a switch
    between slabs and a block table, a call that still passes ODMA_REUSE_PLAN must plan again by itself."""
    lens = np.array([700, 3000, 40], dtype=np.int64)
    w = small_workload(lens, seed=19, bounds=(1024, 4096), large_cap=8192, main=3 * 4096, safety=2 * 8192)
    dp = H.make_pool(w, out_dtype=B.F32, poison=False)
    off, _ = H.assign_perfect(dp, lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(3)]
    H.fill(dp, 0, kv, offsets=off)
    dp.pool.odma_advance(range(3), lens)
    q = wl.queries(w, 0, sharp=True)
    ref = H.oracle_out(w, q, kv)
    H.check(H.decode(dp, 0, q, lens, offsets=off), ref, *TIGHT_F32, what="before migration")
    rc, noff, ncap = dp.pool.odma_migrate(1)
    assert rc == 0 and noff != off[1]
    # the released source slab is overwritten: a stale plan would stream these bytes
    junk = wl.request_kv(w, 0, 1, sharp=True, n_tokens=3000)
    junk = (np.ascontiguousarray(junk[0][::-1]), np.ascontiguousarray(junk[1][::-1]))
    H.fill(dp, 0, [junk], offsets=np.array([off[1]]))
    off2 = off.copy()
    off2[1] = noff
    got = H.decode(dp, 0, q, lens, offsets=off2, flags=B.REUSE_PLAN)
    H.check(got, ref, *TIGHT_F32, what="REUSE_PLAN after migration")
    # same lengths through a block table, flag still set
    bt = wl.shuffled_block_table(lens, w.pool_tokens // 16, 16, seed=20)
    dp2 = H.make_pool(w, out_dtype=B.F32, poison=False)
    off_b, _ = H.assign_perfect(dp2, lens)
    H.fill(dp2, 0, [junk if r == 1 else kv[r] for r in range(3)], offsets=off_b)
    H.decode(dp2, 0, q, lens, offsets=off_b)                          # plans for contiguous slabs
    H.fill(dp2, 0, kv, block_table=bt)
    got = H.decode(dp2, 0, q, lens, block_table=bt, flags=B.REUSE_PLAN)
    H.check(got, ref, *TIGHT_F32, what="REUSE_PLAN after a switch to the paged layout")


def test_fewer_tiles_than_waves_in_a_work_group():
    """Batches with fewer tiles than a work-group has waves: the plan must put the empty ranges on the left (a wave
    waits for its right-hand neighbour's first piece, and an empty wave never hands one over).  One request on one KV
    head growing token by token through 1..3 tiles, both work-group sizes, MQA and two-head pools, all three formats."""
    for kvd, hq, hkv, d, wg in [("bf16", 7, 1, 128, 4), ("bf16", 7, 1, 128, 8), ("bf16", 8, 2, 128, 8),
                                ("bf16", 9, 3, 128, 8), ("bf16", 8, 1, 64, 4), ("fp8", 7, 1, 128, 4),
                                ("fp8", 8, 2, 128, 8)]:
        for n_tok in (1, 16, 17, 31, 32, 33, 48, 49, 64, 65, 96, 97):
            w = small_workload([n_tok], kv_dtype=kvd, hq=hq, hkv=hkv, d=d, seed=hq + n_tok)
            dp = H.make_pool(w, out_dtype=B.F32)
            dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_CU, wg)
            dp.pool.odma_pool_tune(B.TUNE_WAVES_PER_WG, wg)
            off, _ = H.assign_perfect(dp, w.lengths)
            kv = [wl.request_kv(w, 0, 0, sharp=True)]
            H.fill(dp, 0, kv, offsets=off)
            q = wl.queries(w, 0, sharp=True)
            print(f"few tiles: {kvd} hq={hq} hkv={hkv} d={d} wg={wg} len={n_tok}", flush=True)
            got = H.decode(dp, 0, q, w.lengths, offsets=off)
            tol = (1e-4, 1e-2) if kvd == "fp8" else TIGHT_F32
            H.check(got, H.oracle_out(w, q, kv), *tol, what=f"{kvd} hkv={hkv} wg={wg} len={n_tok}")


def test_work_groups_whose_ranges_end_on_segment_ends():
    """Work-groups without a cut leave without the epilogue of the in-kernel merge.  With as many requests as
    work-groups, three KV heads and eight tiles per request and head, every work-group range (24 tiles) begins and ends
    on a segment end while the four waves of a work-group (6 tiles each) still cut segments among themselves; a one-tile
    request in the middle then shifts the second half of the stream, so that the same launch has work-groups with and
    without cuts."""
    n_wg = torch.cuda.get_device_properties(0).multi_processor_count
    rng = np.random.default_rng(21)
    aligned = rng.integers(113, 129, n_wg)                   # 8 tiles of 16 tokens each
    for name, lengths in (("aligned", aligned), ("half shifted", np.concatenate([aligned[:n_wg // 2], [9], aligned[n_wg // 2:]]))):
        w = small_workload(lengths, hq=21, hkv=3, seed=21, bounds=(128, 256, 512), large_cap=512)
        if name == "aligned":
            start, _ = B.odma_stream_plan_ranges(int(sum((l + 15) // 16 for l in lengths)) * 3, n_wg * 4)
            assert all(start[4 * b] % 8 == 0 for b in range(n_wg + 1)), "the case no longer aligns with the plan's shares"
        dp = H.make_pool(w, out_dtype=B.F32)
        pin_launch_shape(dp)
        off, _ = H.assign_perfect(dp, w.lengths)
        kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(w.n_requests)]
        H.fill(dp, 0, kv, offsets=off)
        q = wl.queries(w, 0, sharp=True)
        print(f"no-cut work-groups: {name}, {w.n_requests} requests", flush=True)
        got = H.decode(dp, 0, q, w.lengths, offsets=off)
        H.check(got, H.oracle_out(w, q, kv), *TIGHT_F32, what=name)


def test_device_call_argument_errors():
    w = small_workload([10], seed=10)
    dp = H.make_pool(w)
    h = dp.pool._h
    q = torch.zeros(1, 28, 128, dtype=torch.int16, device=H.DEV)
    assert B.lib.odma_decode_attention(h, 1, 1, q.data_ptr(), None, None, None, 0, q.data_ptr(), 0, None) == B.INVALID_ARG
    assert B.lib.odma_decode_attention(h, 0, 2, q.data_ptr(), q.data_ptr(), q.data_ptr(), None, 0, q.data_ptr(), 0,
                                       None) == B.INVALID_ARG        # n > max_requests
    assert B.lib.odma_gather_kv(h, 0, 8, 4, None, q.data_ptr(), q.data_ptr(), None) == B.INVALID_ARG   # unaligned
    assert B.lib.odma_gather_kv(h, 0, w.pool_tokens, 16, None, q.data_ptr(), q.data_ptr(), None) == B.INVALID_ARG


# ---- config 5: drifting arrivals, recalibration, pre-emptive routing and migration under decode ------------

def test_config5_drift_run_short():
    """Drift run scaled down (64 slots, 160 steps, lengths clipped to 16384, recalibration every 20
    steps, window 128) so the CPU oracle keeps up.  Every host decision is compared with the allocator
    oracle bit for bit; attention (fused odma_decode_step) is compared with the attention oracle on
    all live requests every 16 steps and at every step in which a migration happened."""
    slots, steps, clip = 64, 160, 16384
    w = wl.Workload("drift", 1, 28, 4, 128, "bf16", np.zeros(slots, np.int64), (512, 1024, 2048, 4096),
                    main_tokens=1 << 18, safety_tokens=6 * clip, large_cap=clip, data_seed=555,
                    data_scale=1.0 / math.sqrt(128.0))
    dp = H.make_pool(w, out_dtype=B.F32, max_requests=slots, window=128)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries, max_requests=slots,
                     window=128)
    gen = wl.drift_arrivals(seed=5, n_steps=steps, clip=clip)
    next(gen)
    live = {}                                   # slot -> dict(total, have, k, v)
    serial = 0
    done, checked, migrations, routed = [], 0, 0, 0
    for step in range(steps):
        migrated_now = False
        # admit into free slots
        for s in range(slots):
            if s in live:
                continue
            a = gen.send(step)
            u = np.array([a.uncertainty], np.float32)
            rc, bk, off, cap, st = dp.pool.odma_assign([s], [a.pred_len], u)
            assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(
                map(list, sim.assign([s], [a.pred_len], [u[0]])))
            if st[0] != 0:
                continue
            routed += int(bk[0] == 4)
            rng = np.random.default_rng([w.data_seed, serial])
            serial += 1
            k, _ = wl.draw_values(rng, (a.total_len, 4, 128), 1.0, "bf16")          # sharp keys
            v, _ = wl.draw_values(rng, (a.total_len, 4, 128), w.data_scale, "bf16")
            rc, ov, _ = dp.pool.odma_advance([s], [a.prefilled]); sov, _ = sim.advance([s], [a.prefilled])
            assert ov.tolist() == sov
            if ov[0]:                              # the prompt alone overflows an under-predicted bucket
                assert dp.pool.odma_migrate(s) == sim.migrate(s)[:3]
                assert dp.pool.odma_advance([s], [a.prefilled])[1].tolist() == sim.advance([s], [a.prefilled])[0] == [0]
                migrations += 1
            o, _, _ = dp.pool.odma_pool_lookup([s])
            H.fill(dp, 0, [(k[:a.prefilled], v[:a.prefilled])], offsets=o)
            live[s] = dict(total=a.total_len, have=a.prefilled, k=k, v=v)
        ids = sorted(live)
        # bookkeeping of this step's token, migrating what overflows
        rc, ov, _ = dp.pool.odma_advance(ids); sov, _ = sim.advance(ids)
        assert ov.tolist() == sov
        stopped = []
        for s, o in zip(ids, ov):
            if not o:
                continue
            got, want = dp.pool.odma_migrate(s), sim.migrate(s)
            assert got == want[:3]
            if got[0] == 0:
                migrations += 1
                migrated_now = True
                assert dp.pool.odma_advance([s])[1].tolist() == sim.advance([s])[0] == [0]
            else:
                stopped.append(s)                  # already at L_max (or safety pool full): generation stops
        ids = [s for s in ids if s not in stopped]
        off, ln, _ = dp.pool.odma_pool_lookup(ids)
        assert ln.tolist() == [live[s]["have"] + 1 for s in ids]
        k_new = np.stack([live[s]["k"][live[s]["have"]] for s in ids])
        v_new = np.stack([live[s]["v"][live[s]["have"]] for s in ids])
        rngq = np.random.default_rng([w.data_seed, 7, step])
        q, _ = wl.draw_values(rngq, (len(ids), 28, 128), 1.0, "bf16")
        got = H.decode_step(dp, 0, q, k_new, v_new, ln, offsets=off)
        for s in ids:
            live[s]["have"] += 1
        if step % 16 == 0 or migrated_now:
            ref = H.oracle_out(w, q, [(live[s]["k"][:live[s]["have"]], live[s]["v"][:live[s]["have"]]) for s in ids])
            H.check(got, ref, *TIGHT_F32, what=f"drift step {step}")
            checked += 1
        fin = [s for s in sorted(live) if live[s]["have"] >= live[s]["total"] or s in stopped]
        if fin:
            done += [live[s]["have"] for s in fin]
            assert dp.pool.odma_release(fin)[1].tolist() == sim.release(fin)
            for s in fin:
                del live[s]
        if step % 20 == 19:
            assert dp.pool.odma_recalibrate(done) == tuple(sim.recalibrate(done))
            done = []
    st = dp.pool.odma_pool_stats()
    assert st["migrations"] == sim.n_migrations == migrations and st["recalibrations"] == sim.n_recalibrations >= 7
    assert st["done_actual"] == sim.done_actual and st["done_reserved"] == sim.done_reserved
    assert dp.pool.odma_pool_snapshot()[0] == [tuple(r) for r in sim.snapshot()]
    assert checked >= 10 and st["done_requests"] > 50
    util = st["done_actual"] / st["done_reserved"]
    print(f"drift: {st['done_requests']} completed, {migrations} migrations, {routed} routed to the Large Bucket, "
          f"utilization {util:.3f}, boundaries {dp.pool.odma_pool_snapshot()[1]}")


def test_adaptive_loop_script_device_mode():
    """adaptive_loop.py --device: admission, prefill appends, fused decode steps, migrations and background
    recalibration together on the GPU (values are not checked here: test_config5_drift_run_short does that)."""
    import json, os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    cmd = [sys.executable, os.path.join(root, "adaptive_loop.py"), "--device", "--policies", "odma", "--requests", "1500",
           "--budget-tokens", str(1 << 20), "--l-max", "8192", "--safety-slabs", "16", "--window", "500", "--refresh", "100",
           "--max-live", "1024"]
    out = subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=300, cwd=root).stdout
    r = json.loads(out.strip().splitlines()[-1])["policies"][0]
    assert r["requests"] == 1500 and r["recalibrations"] == 15
    d = r["device"]
    assert d["kv_bytes_total"] > 0 and d["decode_ms_total"] > 0 and d["sustained_kv_GBps"] > 100
    assert abs(d["mean_batch"] - r["mean_resident_requests"]) < 0.1 * r["mean_resident_requests"] + 1


# ---- head_dim 64 on the matrix-core path --------------------------------------------------------------

@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("out_dtype", [B.F32, B.BF16])
def test_head_dim_64_matrix_core_path(paged, out_dtype):
    """bf16 pools with head_dim 64 stream two 2 KiB blocks per tile: ragged and degenerate lengths, a long request that
    spans many work-groups, several group sizes, the unfused decode step, and agreement with the vector-ALU kernel."""
    lens = [0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 127, 128, 129, 255, 256, 257, 0, 1000, 1024, 4096, 3]
    for sharp in (False, True):
        w = small_workload(lens, d=64, hq=32, hkv=4, seed=61)
        rel, got, dp = run_case(w, out_dtype=out_dtype, sharp=sharp, paged=paged)
        assert dp.pool.odma_pool_decode_kernel() == B.KERNEL_MFMA
        assert (got[0] == 0).all() and (got[21] == 0).all()
        k, v = wl.request_kv(w, 0, 1, sharp=sharp)
        for h in range(32):                                            # one token: that value row exactly
            np.testing.assert_array_equal(got[1, h], wl.bf16_bits_to_f32(v[0, h // 8]))
    w = small_workload([70000, 17, 333, 2100], d=64, hq=16, hkv=2, seed=62, bounds=(1024, 4096, 16384), large_cap=81920,
                       main=81920 + 4 * 16384, safety=81920)
    _, got_m, _ = run_case(w, out_dtype=out_dtype, sharp=True, paged=paged)
    _, got_v, _ = run_case(w, kernel=B.KERNEL_VALU, out_dtype=out_dtype, sharp=True, paged=paged)
    a, r = tight(out_dtype)
    H.check(got_m, got_v.astype(np.float64), 2 * a, 2 * r, what="head_dim 64: matrix-core vs vector-ALU kernel")
    for hq, hkv in [(4, 4), (16, 1), (6, 2)]:
        run_case(small_workload([333, 5, 2049], d=64, hq=hq, hkv=hkv, seed=hq), out_dtype=out_dtype, sharp=True, paged=paged)


def test_head_dim_64_decode_step_and_launch_shapes():
    lens = np.array([300, 15, 16, 31, 32, 0, 1000, 5000], dtype=np.int64)
    w = small_workload(lens + 1, d=64, hq=32, hkv=4, seed=63, bounds=(1024, 4096, 8192), large_cap=8192)
    n = len(lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
    held = [(k[:-1], v[:-1]) for k, v in kv]
    k_new = np.stack([k[-1] for k, _ in kv]); v_new = np.stack([v[-1] for _, v in kv])
    q = wl.queries(w, 0, sharp=True)
    ref = H.oracle_out(w, q, kv)
    shapes = [dict(), dict(cu=8, wg=8), dict(cu=8, wg=4, depth=3), dict(cu=1, wg=4), dict(cu=4, wg=4, fuse=1)]
    for paged in (False, True):
        for shape in shapes:
            dp = H.make_pool(w, out_dtype=B.F32)
            for knob, key in ((B.TUNE_WAVES_PER_CU, "cu"), (B.TUNE_WAVES_PER_WG, "wg"), (B.TUNE_PIPELINE_DEPTH, "depth"),
                              (B.TUNE_FUSE_REDUCE, "fuse")):
                if key in shape:
                    dp.pool.odma_pool_tune(knob, shape[key])
            if paged:
                where = dict(block_table=wl.shuffled_block_table(lens + 1, w.pool_tokens // 16, 16, seed=64))
            else:
                where = dict(offsets=H.assign_perfect(dp, lens + 1)[0])
            H.fill(dp, 0, held, **where)
            got = H.decode_step(dp, 0, q, k_new, v_new, lens + 1, **where)
            H.check(got, ref, *TIGHT_F32, what=f"head_dim 64 decode step paged={paged} {shape}")
            np.testing.assert_array_equal(got, H.decode(dp, 0, q, lens + 1, **where))


@pytest.mark.parametrize("paged", [False, True])
def test_head_dim_64_fused_decode_steps_across_block_and_tile_boundaries(paged):
    """odma_decode_step with head_dim 64 (the append is fused into the attention launch): 36 steps from lengths around the
    16-token block and 32-token tile boundaries, every step against the oracle, then the pools read back bit for bit."""
    lens0 = np.array([0, 1, 14, 15, 16, 17, 30, 31, 32, 33, 47, 48, 200, 3000, 555], dtype=np.int64)
    steps = 36
    w = small_workload(lens0 + steps, d=64, hq=32, hkv=4, seed=65)
    dp = H.make_pool(w, out_dtype=B.F32)
    assert dp.pool.odma_pool_decode_kernel() == B.KERNEL_MFMA
    n = len(lens0)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
    held = [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)]
    bt = off = None
    if paged:
        bt = wl.shuffled_block_table(lens0 + steps, w.pool_tokens // 16, 16, seed=66)
        H.fill(dp, 0, held, block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, lens0, extra=steps)
        H.fill(dp, 0, held, offsets=off)
    lens = lens0.copy()
    for s in range(steps):
        k_new = np.stack([kv[r][0][lens[r]] for r in range(n)])
        v_new = np.stack([kv[r][1][lens[r]] for r in range(n)])
        lens += 1
        q = wl.queries(w, 0, step=s, sharp=True)
        got = H.decode_step(dp, 0, q, k_new, v_new, lens, offsets=off, block_table=bt)
        ref = H.oracle_out(w, q, [(kv[r][0][:lens[r]], kv[r][1][:lens[r]]) for r in range(n)])
        H.check(got, ref, *TIGHT_F32, what=f"head_dim 64 fused step {s} paged={paged}")
    for r in range(n):
        gk, gv = H.gather(dp, 0, 0 if paged else int(off[r]), int(lens[r]), block_row=bt[r] if paged else None)
        np.testing.assert_array_equal(gk, kv[r][0][:lens[r]]); np.testing.assert_array_equal(gv, kv[r][1][:lens[r]])


# ---- measurement aids -------------------------------------------------------------------------------------------

def test_read_probes_run_and_reject_bad_arguments():
    """The two read probes (linear sweep; 4 KiB blocks through a table) launch, finish and leave their sink alone;
    null pointers and empty sizes come back as ODMA_INVALID_ARG."""
    n_blocks = 3000
    k = torch.ones(n_blocks * 4096, dtype=torch.uint8, device=H.DEV)
    v = torch.ones(n_blocks * 4096, dtype=torch.uint8, device=H.DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    B.odma_stream_read_probe(k, k.numel(), sink)
    for table in (np.arange(n_blocks), np.random.default_rng(5).permutation(n_blocks), np.array([7]), np.arange(1025)):
        t = torch.from_numpy(table.astype(np.int32)).to(H.DEV)
        B.odma_block_read_probe(k, v, t, len(table), sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    t = torch.zeros(4, dtype=torch.int32, device=H.DEV)
    for args in ((None, v, t, 4, sink), (k, None, t, 4, sink), (k, v, None, 4, sink), (k, v, t, 0, sink), (k, v, t, 4, None)):
        with pytest.raises(B.OdmaError) as e:
            B.odma_block_read_probe(*args)
        assert e.value.code == B.INVALID_ARG
    with pytest.raises(B.OdmaError):
        B.odma_stream_read_probe(k, 0, sink)


# ---- large pools: byte offsets past 2^31 inside one KV-head plane ----------------------------------------

def test_offsets_beyond_two_gib_in_a_plane():
    """A 10 M-token pool (2.56 GB per KV-head plane in bf16): slabs and paged blocks near its end are addressed with
    64-bit byte offsets by append, export, decode (both layouts) and prefill."""
    pool_tokens = 10_000_000 // 16 * 16
    lens = np.array([700, 33, 2049], dtype=np.int64)
    w = wl.Workload("big", 1, 4, 1, 128, "bf16", lens, (4096,), main_tokens=pool_tokens - 8192, safety_tokens=8192,
                    large_cap=8192, data_seed=77, data_scale=1.0 / math.sqrt(128))
    dp = H.make_pool(w, out_dtype=B.F32, poison=False)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(3)]
    q = wl.queries(w, 0, sharp=True)
    ref = H.oracle_out(w, q, kv)
    off = np.array([0, 9_000_000 // 16 * 16, pool_tokens - 4096], dtype=np.int64)      # byte offsets 0, 2.3 GB, 2.56 GB
    H.fill(dp, 0, kv, offsets=off)
    H.check(H.decode(dp, 0, q, lens, offsets=off), ref, *TIGHT_F32, what="far slabs")
    gk, gv = H.gather(dp, 0, int(off[2]), int(lens[2]))
    np.testing.assert_array_equal(gk, kv[2][0]); np.testing.assert_array_equal(gv, kv[2][1])
    # paged: block ids drawn from the top of the pool
    n_blocks = pool_tokens // 16
    rng = np.random.default_rng(78)
    ids = n_blocks - 1 - rng.permutation(4096)[:int(((lens + 15) // 16).sum())]
    bt = np.zeros((3, 129), np.int32)
    at = 0
    for r in range(3):
        nb = int((lens[r] + 15) // 16)
        bt[r, :nb] = ids[at:at + nb]
        at += nb
    H.fill(dp, 0, kv, block_table=bt)
    H.check(H.decode(dp, 0, q, lens, block_table=bt), ref, *TIGHT_F32, what="far blocks")
    # prefill of the last 100 tokens of the far slab (request 2 was overwritten by blocks above: refill it)
    H.fill(dp, 0, [kv[2]], offsets=off[2:])
    q_rows, _ = wl.draw_values(rng, (100, 4, 128), 1.0, "bf16")
    got = H.prefill(dp, 0, q_rows, [0], [100], lens[2:], offsets=off[2:])
    from oracle import attention as oa
    H.check(got, oa.attend_chunk(q_rows, kv[2][0], kv[2][1], 1.0 / math.sqrt(128)), what="prefill on a far slab")
