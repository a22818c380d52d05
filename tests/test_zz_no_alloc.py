"""odma_decode_attention_static (the entry point for callers that cannot allocate: static device scratch instead of
the pool's workspace) against odma_decode_attention, through the C ABI.

Same kernels, same plan arithmetic, so the outputs must be equal bit for bit; the oracle bounds both.  Two calls in a
row on the same GPU share the scratch, the second with a smaller batch; then the limits are refused with an error.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from paper_2512_09427_amd import binding as B
from tests import harness as H
from tests.test_gpu_parity import TIGHT_F32, small_workload

pytestmark = pytest.mark.gpu


def _static_decode(dp, q, lengths, *, offsets=None, block_table=None, flags=0):
    n = q.shape[0]
    out = torch.full((n, dp.w.n_q_heads, dp.w.head_dim), float("nan"), dtype=torch.float32, device=H.DEV)
    bt = None if block_table is None else H.to_dev(block_table.astype(np.int32))
    dp.pool.odma_decode_attention_static(0, n, H.to_dev(q), None if offsets is None else H.to_dev(np.asarray(offsets, np.int64)),
                                         H.to_dev(np.asarray(lengths, np.int32)), bt,
                                         0 if bt is None else block_table.shape[1], out, flags)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _case(lens, seed, kv_dtype="bf16", paged=False):
    lens = np.asarray(lens, dtype=np.int64)
    w = small_workload(lens, kv_dtype=kv_dtype, seed=seed, bounds=(1024, 8192, 32768), large_cap=32768)
    dp = H.make_pool(w, out_dtype=B.F32)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(len(lens))]
    q = wl.queries(w, 0, sharp=True)
    if paged:
        where = dict(block_table=wl.shuffled_block_table(lens, w.pool_tokens // 16, 16, seed=seed))
    else:
        where = dict(offsets=H.assign_perfect(dp, np.maximum(lens, 1))[0])
    H.fill(dp, 0, kv, **where)
    ref = H.oracle_out(w, q, kv)
    ref[lens == 0] = 0.0
    return dp, q, lens, where, ref


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    # first call: a batch whose long request is cut over tens of work-groups (partials, counters and merges in use)
    dp1, q1, lens1, where1, ref1 = _case([32768, 0, 129, 5000, 64, 0, 9000, 1, 700, 17], seed=51)
    # second call: a smaller batch of another pool on the same GPU (same scratch, stale contents of the first call)
    dp2, q2, lens2, where2, ref2 = _case([300, 31, 2100], seed=52)
    for rounds in range(2):
        print(f"static entry point, round {rounds}: large batch", flush=True)
        want1 = H.decode(dp1, 0, q1, lens1, **where1)
        got1 = _static_decode(dp1, q1, lens1, **where1)
        np.testing.assert_array_equal(got1, want1)
        H.check(got1, ref1, *TIGHT_F32, what="static scratch, large batch")
        print(f"static entry point, round {rounds}: smaller batch", flush=True)
        want2 = H.decode(dp2, 0, q2, lens2, **where2)
        got2 = _static_decode(dp2, q2, lens2, **where2)
        np.testing.assert_array_equal(got2, want2)
        H.check(got2, ref2, *TIGHT_F32, what="static scratch, smaller batch")
        # a plan left by another pool must not be reused even when the flag asks for it
        again1 = _static_decode(dp1, q1, lens1, flags=B.REUSE_PLAN, **where1)
        np.testing.assert_array_equal(again1, want1)
        # and one left by this pool in this state may be
        again1 = _static_decode(dp1, q1, lens1, flags=B.REUSE_PLAN, **where1)
        np.testing.assert_array_equal(again1, want1)


def test_static_scratch_entry_point_paged_and_fp8():
    dp, q, lens, where, ref = _case([4000, 16, 333, 0, 47], seed=53, paged=True)
    got = _static_decode(dp, q, lens, **where)
    np.testing.assert_array_equal(got, H.decode(dp, 0, q, lens, **where))
    H.check(got, ref, *TIGHT_F32, what="static scratch, paged")
    dp, q, lens, where, ref = _case([2500, 33, 1], seed=54, kv_dtype="fp8")
    got = _static_decode(dp, q, lens, **where)
    np.testing.assert_array_equal(got, H.decode(dp, 0, q, lens, **where))
    H.check(got, ref, 1e-4, 1e-2, what="static scratch, fp8 pools")


def test_static_scratch_entry_point_needs_no_workspace_and_refuses_what_does_not_fit():
    lens = np.array([200, 40], dtype=np.int64)
    w = small_workload(lens, seed=55)
    kvd = B.BF16
    elems = w.n_kv_heads * w.pool_tokens * w.head_dim
    k_pool = torch.zeros(elems, dtype=torch.int16, device=H.DEV)
    v_pool = torch.zeros(elems, dtype=torch.int16, device=H.DEV)
    args = dict(n_layers=1, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, kv_dtype=kvd,
                out_dtype=B.F32, main_tokens=w.main_tokens, safety_tokens=w.safety_tokens, large_cap=w.large_cap,
                boundaries=w.boundaries, max_requests=2000, align_tokens=w.align_tokens)
    cfg, keep = B.make_config(**args, k_pool=k_pool, v_pool=v_pool, workspace=None)
    pool = B.Pool(cfg, keep)
    dp = H.DevicePool(pool, k_pool, v_pool, None, w, B.F32)
    off, _ = H.assign_perfect(dp, lens)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(2)]
    H.fill(dp, 0, kv, offsets=off)
    q = wl.queries(w, 0, sharp=True)
    got = _static_decode(dp, q, lens, offsets=off)
    H.check(got, H.oracle_out(w, q, kv), *TIGHT_F32, what="static scratch, pool without a workspace")
    # the workspace entry point refuses this pool; the static one refuses what exceeds its limits
    out = torch.zeros(2, w.n_q_heads, w.head_dim, dtype=torch.float32, device=H.DEV)
    qd, od, ld = H.to_dev(q), H.to_dev(np.asarray(off, np.int64)), H.to_dev(lens.astype(np.int32))
    h = pool._h
    assert B.lib.odma_decode_attention(h, 0, 2, qd.data_ptr(), od.data_ptr(), ld.data_ptr(), None, 0, out.data_ptr(), 0,
                                       None) == B.INVALID_ARG
    assert B.lib.odma_decode_attention_static(h, 0, 1025, qd.data_ptr(), od.data_ptr(), ld.data_ptr(), None, 0,
                                              out.data_ptr(), 0, None) == B.INVALID_ARG
    assert "ODMA_STATIC_MAX_REQUESTS" in B.odma_last_error()
    assert B.lib.odma_decode_attention_static(h, 0, 2, qd.data_ptr(), od.data_ptr(), ld.data_ptr(), None, 0,
                                              out.data_ptr(), B.SKIP_REDUCE, None) == B.INVALID_ARG
    pool.odma_pool_tune(B.TUNE_WAVES_PER_CU, 16)                      # 1024 four-wave work-groups on 256 CUs
    assert B.lib.odma_decode_attention_static(h, 0, 2, qd.data_ptr(), od.data_ptr(), ld.data_ptr(), None, 0,
                                              out.data_ptr(), 0, None) == B.INVALID_ARG
    assert "work-groups" in B.odma_last_error()
    torch.cuda.synchronize()
