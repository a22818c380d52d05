"""GPU parity for odma_prefill_attention (causal attention of the last n_q tokens of each request over its slab)
against the oracle's attend_chunk, through the C ABI.

Tolerance: the stated bf16-in / fp32-accumulate bound |gpu - oracle| <= 2e-3 + 1e-2 |oracle|, and on top the
engineering bound of this kernel: inputs are exact bf16, scores are exact products accumulated in fp32, and each
softmax weight is rounded once to bf16 for the P V product (8 significant bits: at most 2^-8 relative), so
|gpu - oracle| <= 2^-8 * sum_t p_t |v_t|  +  2e-5 + 2e-4 |oracle|   (fp32 output; + 2^-8 |oracle| for bf16 output),
where the first term is the oracle's own attention over |V| (same weights).
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as oa
from paper_2512_09427_amd import binding as B
from tests import harness as H
from tests.test_gpu_parity import small_workload

pytestmark = pytest.mark.gpu

TIGHT = (2e-5, 2e-4)
P_ROUNDING = 2.0 ** -8


def chunk_case(lens, n_q, *, paged=False, sharp=False, hq=28, hkv=4, seed=0, shuffle_rows=False, out_dtype=B.F32,
               pad_rows=0, column_tiles=0, kv_dtype="bf16", **kw):
    """Requests hold lens[r] tokens, the last n_q[r] of them carry queries.  Returns (got, ref, dp, q_start)."""
    lens, n_q = np.asarray(lens, np.int64), np.asarray(n_q, np.int64)
    w = small_workload(lens, kv_dtype=kv_dtype, hq=hq, hkv=hkv, seed=seed, **kw)
    dp = H.make_pool(w, out_dtype=out_dtype)
    dp.pool.odma_pool_tune(B.TUNE_PREFILL_COLUMN_TILES, column_tiles)
    # fp8 pools hold value / FP8_SCALE: the K factor joins the softmax scale, the V factor the output
    f = wl.FP8_SCALE if kv_dtype == "fp8" else 1.0
    sign_off = 0x7f if kv_dtype == "fp8" else 0x7fff
    n = len(lens)
    kv = [wl.request_kv(w, 0, r, sharp=sharp) for r in range(n)]
    rng = np.random.default_rng(500 + seed)
    total = int(n_q.sum()) + pad_rows
    scale = 1.0 if sharp else w.data_scale
    q_rows, _ = wl.draw_values(rng, (total, hq, 128), scale, "bf16")
    order = rng.permutation(n) if shuffle_rows else np.arange(n)
    q_start = np.zeros(n, np.int64)
    at = 0
    for r in order:                                                    # request r's rows sit at q_start[r] ..
        q_start[r] = at
        at += int(n_q[r])
    if paged:
        bt = wl.shuffled_block_table(lens, w.pool_tokens // 16, 16, seed=79)
        H.fill(dp, 0, kv, block_table=bt)
        got = H.prefill(dp, 0, q_rows, q_start, n_q, lens, block_table=bt)
    else:
        off, _ = H.assign_perfect(dp, lens)
        H.fill(dp, 0, kv, offsets=off)
        got = H.prefill(dp, 0, q_rows, q_start, n_q, lens, offsets=off)
    ref = np.full((total, hq, 128), np.nan)
    ref_abs = np.zeros((total, hq, 128))
    for r in range(n):
        s, c = int(q_start[r]), int(n_q[r])
        ref[s:s + c] = oa.attend_chunk(q_rows[s:s + c], kv[r][0], kv[r][1], f / np.sqrt(128.0)) * f
        ref_abs[s:s + c] = oa.attend_chunk(q_rows[s:s + c], kv[r][0], kv[r][1] & sign_off, f / np.sqrt(128.0)) * f
    written = ~np.isnan(ref[:, 0, 0])
    assert np.isnan(got[~written]).all()                               # rows of nobody stay untouched
    what = f"prefill paged={paged} sharp={sharp}"
    H.check(got[written], ref[written], what=what)
    a, rel = TIGHT
    if out_dtype == B.BF16:
        rel += 2.0 ** -8
    err = H.check(got[written], ref[written], a + P_ROUNDING * ref_abs[written], rel, what=what + " (tight)")
    return err, got, ref, dp, kv, q_rows, q_start


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("sharp", [False, True])
@pytest.mark.parametrize("column_tiles", [2, 4])
def test_whole_prompts_of_ragged_lengths(paged, sharp, column_tiles):
    lens = [1, 2, 15, 16, 17, 37, 100, 0, 333, 1000, 64, 255]
    err, *_ = chunk_case(lens, lens, paged=paged, sharp=sharp, seed=1, column_tiles=column_tiles)
    print(f"prefill whole prompts paged={paged} sharp={sharp}: max err / max|ref| = {err:.2e}")


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("column_tiles", [2, 4])
def test_chunks_of_longer_requests_in_any_row_order(paged, column_tiles):
    lens = [700, 64, 1500, 16, 333, 2048, 90, 5]
    n_q = [300, 0, 17, 16, 1, 512, 90, 2]
    err, got, ref, dp, kv, q_rows, q_start = chunk_case(lens, n_q, paged=paged, sharp=True, seed=2, shuffle_rows=True,
                                                        pad_rows=3, column_tiles=column_tiles)
    print(f"prefill chunks paged={paged}: max err / max|ref| = {err:.2e}")


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("column_tiles", [2, 4])
def test_prefill_on_fp8_pools(paged, column_tiles):
    """E4M3 pools: the loader waves widen K/V to bf16 on the way into LDS (exact), the rest of the kernel is shared;
    k_scale joins the softmax scale and v_scale the output.  Same bound as on bf16 pools."""
    lens = [700, 64, 1500, 16, 333, 2048, 90, 5, 1, 17, 31, 33]
    n_q = [300, 0, 17, 16, 333, 512, 90, 2, 1, 17, 31, 20]
    for sharp in (False, True):
        err, *_ = chunk_case(lens, n_q, paged=paged, sharp=sharp, seed=31, shuffle_rows=True, column_tiles=column_tiles,
                             kv_dtype="fp8")
        print(f"prefill on fp8 pools paged={paged} sharp={sharp}: max err / max|ref| = {err:.2e}")


def test_last_row_of_a_chunk_is_the_decode_query():
    """The chunk's last token sees the whole slab: the same answer as odma_decode_attention for that query."""
    lens = np.array([129, 500, 31, 1024])
    n_q = np.array([40, 1, 31, 200])
    _, got, ref, dp, kv, q_rows, q_start = chunk_case(lens, n_q, sharp=True, seed=3)
    last = q_start + n_q - 1
    w = dp.w
    dp2 = H.make_pool(w, out_dtype=B.F32)
    off, _ = H.assign_perfect(dp2, lens)
    H.fill(dp2, 0, kv, offsets=off)
    dec = H.decode(dp2, 0, q_rows[last], lens, offsets=off)
    H.check(got[last], dec.astype(np.float64), 1e-3, 2e-4, what="prefill last row vs decode")


def test_other_group_sizes_bf16_output_and_row_clamp():
    for hq, hkv in [(4, 4), (16, 1), (32, 2), (8, 2), (12, 4)]:
        for column_tiles in (2, 4):
            chunk_case([333, 5, 70], [100, 5, 70], sharp=True, hq=hq, hkv=hkv, seed=hq, column_tiles=column_tiles)
    chunk_case([400, 33], [400, 20], sharp=True, out_dtype=B.BF16, seed=4)
    # total_q smaller than the rows the requests name: the surplus rows are neither read nor written
    lens, n_q = np.array([50, 60]), np.array([50, 60])
    w = small_workload(lens, seed=5)
    dp = H.make_pool(w, out_dtype=B.F32)
    kv = [wl.request_kv(w, 0, r, sharp=True) for r in range(2)]
    off, _ = H.assign_perfect(dp, lens)
    H.fill(dp, 0, kv, offsets=off)
    q_rows, _ = wl.draw_values(np.random.default_rng(6), (110, 28, 128), 1.0, "bf16")
    got = H.prefill(dp, 0, q_rows, [0, 50], n_q, lens, offsets=off, total_q=80)
    assert np.isnan(got[80:]).all() and np.isfinite(got[:80]).all()
    # request 1 is treated as holding 30 query rows: the last 30 of its 60 tokens
    ref = oa.attend_chunk(q_rows[50:80], kv[1][0], kv[1][1], 1.0 / np.sqrt(128.0))
    H.check(got[50:80], ref, 1e-3, 2e-4, what="clamped rows")


def test_long_prompt_and_many_requests():
    rng = np.random.default_rng(8)
    lens = np.concatenate([[6000], rng.integers(1, 300, 40)])
    n_q = np.concatenate([[1500], lens[1:]])
    for column_tiles in (2, 4):
        err, *_ = chunk_case(lens, n_q, sharp=True, seed=7, bounds=(1024, 4096, 8192), large_cap=8192, column_tiles=column_tiles)
        print(f"prefill long prompt + 40 short, {column_tiles} column tiles: max err / max|ref| = {err:.2e}")


def test_prefill_needs_the_matrix_core_path():
    w = wl.tiny()
    dp = H.make_pool(w)
    z = torch.zeros(4, dtype=torch.int64, device=H.DEV)
    with pytest.raises(B.OdmaError):
        dp.pool.odma_prefill_attention(0, 1, z, 1, z, z, z, z, None, 0, z)


@pytest.mark.parametrize("gain", [3.0, 5.0])
@pytest.mark.parametrize("column_tiles", [2, 4])
def test_scores_that_outgrow_the_first_pair_are_redone_with_moving_references(gain, column_tiles):
    """The fast pass fixes each column's softmax reference on the first 32 tokens.  Here every later key scores
    about 100 (gain 3) or 165 (gain 5: past the fp32 exponent range) exponent units above them, so the weight sums
    blow up and the work-group repeats the item with the online softmax that moves its references."""
    n_tok, hq, hkv = 200, 28, 4
    w = small_workload([n_tok], seed=11)
    dp = H.make_pool(w, out_dtype=B.F32)
    dp.pool.odma_pool_tune(B.TUNE_PREFILL_COLUMN_TILES, column_tiles)
    rng = np.random.default_rng(12)
    u = rng.choice([-2.0, 2.0], size=128).astype(np.float32)
    amp = np.where(np.arange(n_tok) < 64, 0.0, gain + (np.arange(n_tok) % 7) * 0.125).astype(np.float32)
    k = wl.f32_to_bf16_bits(np.broadcast_to((amp[:, None] * u[None, :] / 2)[:, None, :], (n_tok, hkv, 128)).copy())
    v, _ = wl.draw_values(rng, (n_tok, hkv, 128), 1.0, "bf16")
    q = wl.f32_to_bf16_bits(np.broadcast_to(u, (n_tok, hq, 128)).copy())
    off, _ = H.assign_perfect(dp, w.lengths)
    H.fill(dp, 0, [(k, v)], offsets=off)
    got = H.prefill(dp, 0, q, [0], [n_tok], [n_tok], offsets=off)
    ref = oa.attend_chunk(q, k, v, 1.0 / np.sqrt(128.0))
    ref_abs = oa.attend_chunk(q, k, v & 0x7fff, 1.0 / np.sqrt(128.0))
    H.check(got, ref, what=f"outgrowing scores, gain {gain}")
    H.check(got, ref, TIGHT[0] + P_ROUNDING * ref_abs, TIGHT[1], what=f"outgrowing scores, gain {gain} (tight)")
    # the rows before the jump are plain means of their visible values, the rows after it ignore the early tokens
    np.testing.assert_allclose(got[10, 0], wl.bf16_bits_to_f32(v[:11, 0]).mean(axis=0), rtol=0, atol=2e-2)


def test_thousands_of_short_prompts():
    """More requests than one search round covers (64 x 64) and many empty ones: the item prefix repeats values and the
    two-round request search has to land on the request that owns the item."""
    rng = np.random.default_rng(21)
    lens = rng.integers(0, 40, 5000).astype(np.int64)
    n_q = np.where(rng.random(5000) < 0.3, 0, np.minimum(lens, rng.integers(0, 40, 5000))).astype(np.int64)
    err, *_ = chunk_case(lens, n_q, sharp=True, seed=22, hq=8, hkv=2, shuffle_rows=True, bounds=(64, 128, 256), large_cap=256)
    print(f"prefill 5000 short prompts: max err / max|ref| = {err:.2e}")
