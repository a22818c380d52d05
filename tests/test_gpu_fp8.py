"""GPU parity for fp8 (OCP E4M3) K/V storage: the matrix-core kernel on one-byte pools against the CPU oracle.

Both sides read the same stored bytes (the oracle widens them through its own table of the 256 E4M3 values), so
what is compared is the kernel's arithmetic on them, not the quantisation of K and V.  That arithmetic is not exact
fp32: the queries and the softmax weights enter the fp8 matrix instructions as a high plus a low E4M3 part, about
8 significant bits each (a bf16's worth).  A score therefore carries a relative error of the order 2^-8 / sqrt(3)
per term, the weights the same again, and the sums average it down; the stated bf16 bound
|gpu - oracle| <= 2e-3 + 1e-2 |oracle| is kept, and the engineering bound asserted on top is
1e-4 + 1e-2 |oracle| for peaked ("sharp") and flat softmax alike.  Bytes are compared bit for bit.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import allocator as al
from paper_2512_09427_amd import binding as B
from tests import harness as H
from tests.test_gpu_parity import pin_launch_shape, small_workload

pytestmark = pytest.mark.gpu

TIGHT_FP8 = (1e-4, 1e-2)


def fp8_case(lens, *, paged=False, sharp=False, out_dtype=B.F32, seed=0, hq=28, hkv=4, tune=(), pin=False, **kw):
    w = small_workload(lens, kv_dtype="fp8", hq=hq, hkv=hkv, seed=seed, **kw)
    dp = H.make_pool(w, out_dtype=out_dtype)
    assert dp.pool.odma_pool_decode_kernel() == B.KERNEL_MFMA
    if pin:
        pin_launch_shape(dp)
    for knob, val in tune:
        dp.pool.odma_pool_tune(knob, val)
    n = w.n_requests
    kv = [wl.request_kv(w, 0, r, sharp=sharp) for r in range(n)]
    q = wl.queries(w, 0, sharp=sharp)
    if paged:
        bt = wl.shuffled_block_table(w.lengths, w.pool_tokens // 16, 16, seed=78)
        H.fill(dp, 0, kv, block_table=bt)
        got = H.decode(dp, 0, q, w.lengths, block_table=bt)
        where = dict(block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, w.lengths)
        H.fill(dp, 0, kv, offsets=off)
        got = H.decode(dp, 0, q, w.lengths, offsets=off)
        where = dict(offsets=off)
    ref = H.oracle_out(w, q, kv)
    what = f"fp8 paged={paged} sharp={sharp}"
    H.check(got, ref, what=what)
    a, r = TIGHT_FP8
    if out_dtype == B.BF16:
        r += 2.0 ** -8
    rel = H.check(got, ref, a, r, what=what + " (tight)")
    return rel, got, dp, w, kv, q, where


RAGGED = [0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 127, 128, 129, 255, 256, 257, 0, 1000, 1024, 4096, 3]


def test_fp8_rows_round_trip_bit_exactly():
    """append -> pool block format -> gather gives the bytes back, contiguous and paged, bulk and one row at a time."""
    lens = [1, 16, 17, 100, 333]
    w = small_workload(lens, kv_dtype="fp8", seed=5)
    kv = [wl.request_kv(w, 0, r) for r in range(len(lens))]
    dp = H.make_pool(w)
    off, _ = H.assign_perfect(dp, w.lengths)
    H.fill(dp, 0, kv, offsets=off)
    for r, n in enumerate(lens):
        gk, gv = H.gather(dp, 0, int(off[r]), n)
        np.testing.assert_array_equal(gk, kv[r][0]); np.testing.assert_array_equal(gv, kv[r][1])
    dp = H.make_pool(w)
    bt = wl.shuffled_block_table(w.lengths, w.pool_tokens // 16, 16, seed=6)
    part = [(k[:-1], v[:-1]) for k, v in kv]
    H.fill(dp, 0, part, block_table=bt)
    H.append_one(dp, 0, np.stack([k[-1] for k, _ in kv]), np.stack([v[-1] for _, v in kv]),
                 np.array(lens) - 1, block_table=bt)
    for r, n in enumerate(lens):
        gk, gv = H.gather(dp, 0, 0, n, block_row=bt[r])
        np.testing.assert_array_equal(gk, kv[r][0]); np.testing.assert_array_equal(gv, kv[r][1])


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("sharp", [False, True])
def test_fp8_ragged_and_degenerate_lengths(paged, sharp):
    rel, got, dp, w, kv, q, _ = fp8_case(RAGGED, paged=paged, sharp=sharp, seed=1)
    assert (got[0] == 0).all() and (got[21] == 0).all()                # empty requests give zeros
    # one token: the weight is exactly 1 and the output is that value row, de-quantised, exactly
    v = wl.e4m3_bits_to_f32(kv[1][1]) * np.float32(wl.FP8_SCALE)
    for h in range(28):
        np.testing.assert_array_equal(got[1, h], v[0, h // 7])
    print(f"fp8 ragged paged={paged} sharp={sharp}: max err / max|ref| = {rel:.2e}")


@pytest.mark.parametrize("out_dtype", [B.BF16, B.F32])
@pytest.mark.parametrize("sharp", [False, True])
def test_fp8_config2_shape(out_dtype, sharp):
    w0 = wl.qwen_b64()
    rel, got_c, *_ = fp8_case(w0.lengths, sharp=sharp, out_dtype=out_dtype, seed=2, bounds=w0.boundaries,
                              large_cap=w0.large_cap, main=w0.main_tokens, safety=w0.safety_tokens, pin=True)
    print(f"fp8 config-2 shape out={out_dtype} sharp={sharp}: max err / max|ref| = {rel:.2e}")
    _, got_p, *_ = fp8_case(w0.lengths, sharp=sharp, out_dtype=out_dtype, seed=2, bounds=w0.boundaries, paged=True,
                            large_cap=w0.large_cap, main=w0.main_tokens, safety=w0.safety_tokens, pin=True)
    np.testing.assert_array_equal(got_c, got_p)                        # layout must not change a single bit


def test_fp8_launch_shapes_group_sizes_and_long_request():
    lens = np.array([2100, 17, 0, 640, 16, 70000, 1, 333, 48, 1279, 15, 4096, 31, 33], dtype=np.int64)
    kw = dict(seed=33, bounds=(1024, 4096, 16384), large_cap=81920, main=81920 + 16 * 16384, safety=81920)
    shapes = [(), ((B.TUNE_WAVES_PER_CU, 8), (B.TUNE_WAVES_PER_WG, 8)), ((B.TUNE_WAVES_PER_CU, 8), (B.TUNE_WAVES_PER_WG, 4)),
              ((B.TUNE_PIPELINE_DEPTH, 3),), ((B.TUNE_WAVES_PER_CU, 1),), ((B.TUNE_FUSE_REDUCE, 1),),
              ((B.TUNE_WAVES_PER_CU, 8), (B.TUNE_WAVES_PER_WG, 8), (B.TUNE_PIPELINE_DEPTH, 3), (B.TUNE_FUSE_REDUCE, 1))]
    for paged in (False, True):
        for tune in shapes:
            fp8_case(lens, paged=paged, sharp=True, tune=tune, **kw)
    for hq, hkv in [(4, 4), (16, 1), (32, 2), (8, 8)]:
        fp8_case([333, 5, 2049], sharp=True, hq=hq, hkv=hkv, seed=hq)


@pytest.mark.parametrize("paged", [False, True])
def test_fp8_fused_decode_steps_across_block_and_tile_boundaries(paged):
    """odma_decode_step on fp8 pools (the append is fused into the attention launch): 36 steps from lengths around the
    16-token block and 32-token tile boundaries; every step against the oracle on len + 1 tokens, and afterwards the
    pools hold exactly the appended bytes (read back through odma_gather_kv)."""
    lens0 = np.array([0, 1, 14, 15, 16, 17, 30, 31, 32, 33, 47, 48, 200, 3000, 555], dtype=np.int64)
    steps = 36
    w = small_workload(lens0 + steps, kv_dtype="fp8", seed=21)
    dp = H.make_pool(w, out_dtype=B.F32)
    n = len(lens0)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
    held = [(k[:lens0[r]], v[:lens0[r]]) for r, (k, v) in enumerate(kv)]
    bt = off = None
    if paged:
        bt = wl.shuffled_block_table(lens0 + steps, w.pool_tokens // 16, 16, seed=22)
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
        H.check(got, ref, *TIGHT_FP8, what=f"fp8 fused step {s} paged={paged}")
    for r in range(n):
        gk, gv = H.gather(dp, 0, 0 if paged else int(off[r]), int(lens[r]), block_row=bt[r] if paged else None)
        np.testing.assert_array_equal(gk, kv[r][0][:lens[r]]); np.testing.assert_array_equal(gv, kv[r][1][:lens[r]])


@pytest.mark.parametrize("shape", [(8, 8, 3), (8, 4, 2), (4, 4, 3), (16, 8, 2)])
def test_fp8_fused_decode_step_launch_shapes(shape):
    """The fused fp8 step under other launch shapes (waves per CU, waves per work-group, register buffers), contiguous
    and paged, with and without the in-kernel merge: the oracle's outputs and the appended bytes."""
    wpc, wpw, nbuf = shape
    lens = np.array([300, 15, 16, 31, 32, 0, 1000, 63, 64, 3000], dtype=np.int64)
    w = small_workload(lens + 1, kv_dtype="fp8", seed=23)
    n = len(lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
    held = [(k[:-1], v[:-1]) for k, v in kv]
    k_new = np.stack([k[-1] for k, _ in kv]); v_new = np.stack([v[-1] for _, v in kv])
    q = wl.queries(w, 0, sharp=True)
    for paged in (False, True):
        for fuse_reduce in (1, 0):
            dp = H.make_pool(w, out_dtype=B.F32)
            pin_launch_shape(dp, wpc, wpw)
            dp.pool.odma_pool_tune(B.TUNE_PIPELINE_DEPTH, nbuf)
            dp.pool.odma_pool_tune(B.TUNE_FUSE_REDUCE, fuse_reduce)
            if paged:
                bt = wl.shuffled_block_table(lens + 1, w.pool_tokens // 16, 16, seed=24)
                where = dict(block_table=bt)
            else:
                off, _ = H.assign_perfect(dp, lens + 1)
                where = dict(offsets=off)
            H.fill(dp, 0, held, **where)
            got = H.decode_step(dp, 0, q, k_new, v_new, lens + 1, **where)
            H.check(got, H.oracle_out(w, q, kv), *TIGHT_FP8, what=f"fp8 fused step shape={shape} paged={paged}")
            for r in (0, 3, 9):
                gk, gv = H.gather(dp, 0, 0 if paged else int(where["offsets"][r]), int(lens[r]) + 1,
                                  block_row=where["block_table"][r] if paged else None)
                np.testing.assert_array_equal(gk, kv[r][0]); np.testing.assert_array_equal(gv, kv[r][1])


def test_fp8_decode_step_appends_then_attends():
    """On fp8 pools odma_decode_step gives the same result as the append followed by the attention call, and the
    appended bytes are in the pool."""
    lens = np.array([300, 15, 16, 31, 32, 0, 1000], dtype=np.int64)
    w = small_workload(lens + 1, kv_dtype="fp8", seed=9)
    n = len(lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(n)]
    held = [(k[:-1], v[:-1]) for k, v in kv]
    k_new = np.stack([k[-1] for k, _ in kv]); v_new = np.stack([v[-1] for _, v in kv])
    q = wl.queries(w, 0, sharp=True)
    for paged in (False, True):
        dp = H.make_pool(w, out_dtype=B.F32)
        if paged:
            bt = wl.shuffled_block_table(lens + 1, w.pool_tokens // 16, 16, seed=10)
            where = dict(block_table=bt)
        else:
            off, _ = H.assign_perfect(dp, lens + 1)
            where = dict(offsets=off)
        H.fill(dp, 0, held, **where)
        got = H.decode_step(dp, 0, q, k_new, v_new, lens + 1, **where)
        H.check(got, H.oracle_out(w, q, kv), *TIGHT_FP8, what=f"fp8 decode step paged={paged}")
        np.testing.assert_array_equal(got, H.decode(dp, 0, q, lens + 1, **where))


def test_fp8_migration_moves_bytes_and_keeps_the_output():
    w = small_workload([300, 500, 64], kv_dtype="fp8", seed=12, bounds=(256, 512, 1024), large_cap=1024)
    dp = H.make_pool(w, out_dtype=B.F32)
    sim = al.PoolSim(w.main_tokens, w.safety_tokens, w.large_cap, boundaries=w.boundaries)
    pred = [100, 500, 64]
    rc, bk, off, cap, st = dp.pool.odma_assign(range(3), pred)
    assert (bk.tolist(), off.tolist(), cap.tolist(), st.tolist()) == tuple(sim.assign(range(3), pred))
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(3)]
    held = int(cap[0])
    first = [(kv[0][0][:held], kv[0][1][:held]), kv[1], kv[2]]
    H.fill(dp, 0, first, offsets=off)
    lens = np.array([held, 500, 64])
    dp.pool.odma_advance(range(3), lens); sim.advance(range(3), lens.tolist())
    q = wl.queries(w, 0, sharp=True)
    before = H.decode(dp, 0, q, lens, offsets=off)
    assert dp.pool.odma_advance([0])[1].tolist() == sim.advance([0])[0] == [1]
    rc, noff, ncap = dp.pool.odma_migrate(0)
    assert (rc, noff, ncap) == sim.migrate(0)[:3]
    torch.cuda.synchronize()
    off2 = off.copy(); off2[0] = noff
    np.testing.assert_array_equal(before, H.decode(dp, 0, q, lens, offsets=off2))
    gk, gv = H.gather(dp, 0, noff, held)
    np.testing.assert_array_equal(gk, kv[0][0][:held]); np.testing.assert_array_equal(gv, kv[0][1][:held])
