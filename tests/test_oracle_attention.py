"""Pins for oracle/attention.py: each checks the oracle against something other
than itself -- scalar brute force, a library routine, closed forms, invariants."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as oa


def brute_force(q, k, v, scale):
    """Scalar triple loop in Python floats (fp64).  q [Hq][D], k/v [T][Hkv][D]."""
    n_q, d = len(q), len(q[0])
    n_t, n_kv = len(k), len(k[0])
    group = n_q // n_kv
    out = [[0.0] * d for _ in range(n_q)]
    for h in range(n_q):
        g = h // group
        s = []
        for t in range(n_t):
            acc = 0.0
            for i in range(d):
                acc += q[h][i] * k[t][g][i]
            s.append(acc * scale)
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = sum(e)
        for i in range(d):
            acc = 0.0
            for t in range(n_t):
                acc += e[t] / z * v[t][g][i]
            out[h][i] = acc
    return np.array(out)


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


# ---- P1: brute force ----------------------------------------------------------

def test_tiny_config_matches_brute_force():
    w = wl.tiny()
    assert w.lengths.tolist() == [69, 73, 101, 123]
    q = wl.queries(w, 0)
    scale = 1.0 / math.sqrt(w.head_dim)
    for r in range(w.n_requests):
        k, v = wl.request_kv(w, 0, r)
        ref = brute_force(q[r].tolist(), k.tolist(), v.tolist(), scale)
        got64 = oa.attend_one(q[r], k, v, scale, np.float64)
        got32 = oa.attend_one(q[r], k, v, scale, np.float32)
        np.testing.assert_allclose(got64, ref, rtol=0, atol=1e-12)
        np.testing.assert_allclose(got32, ref, rtol=0, atol=1e-6)


@pytest.mark.parametrize("seed", range(12))
def test_micro_cases_match_brute_force(seed):
    rng = np.random.default_rng(seed)
    n_kv = int(rng.integers(1, 4))
    group = int(rng.integers(1, 8))
    d = int(rng.choice([8, 16, 32, 64]))
    n_t = int(rng.integers(1, 41))
    q, k, v = _rand(rng, n_kv * group, d), _rand(rng, n_t, n_kv, d), _rand(rng, n_t, n_kv, d)
    scale = float(rng.uniform(0.05, 1.5))
    ref = brute_force(q.tolist(), k.tolist(), v.tolist(), scale)
    np.testing.assert_allclose(oa.attend_one(q, k, v, scale, np.float64), ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oa.attend_one(q, k, v, scale, np.float32), ref, rtol=0, atol=2e-6)


# ---- P2: library special case ---------------------------------------------------

@pytest.mark.parametrize("seed,n_kv,group,d,n_t", [(0, 4, 7, 128, 300), (1, 1, 2, 64, 77), (2, 2, 4, 32, 1)])
def test_matches_torch_sdpa(seed, n_kv, group, d, n_t):
    rng = np.random.default_rng(seed)
    q, k, v = _rand(rng, n_kv * group, d), _rand(rng, n_t, n_kv, d), _rand(rng, n_t, n_kv, d)
    tq = torch.from_numpy(q).double()[None, :, None, :]                        # [1, Hq, 1, D]
    tk = torch.from_numpy(k).double().permute(1, 0, 2).repeat_interleave(group, 0)[None]
    tv = torch.from_numpy(v).double().permute(1, 0, 2).repeat_interleave(group, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    got = oa.attend_one(q, k, v, 1.0 / math.sqrt(d), np.float64)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    got32 = oa.attend_one(q, k, v, 1.0 / math.sqrt(d), np.float32)
    np.testing.assert_allclose(got32, ref, rtol=0, atol=2e-6)


# ---- P3: closed forms -----------------------------------------------------------

def test_single_token_returns_its_value_row():
    rng = np.random.default_rng(3)
    q, k, v = _rand(rng, 6, 16), _rand(rng, 1, 2, 16), _rand(rng, 1, 2, 16)
    out = oa.attend_one(q, k, v, 0.25, np.float32)
    for h in range(6):
        np.testing.assert_array_equal(out[h], v[0, h // 3])


def test_zero_query_and_equal_keys_give_mean_of_values():
    rng = np.random.default_rng(4)
    k, v = _rand(rng, 37, 2, 16), _rand(rng, 37, 2, 16)
    out = oa.attend_one(np.zeros((4, 16), np.float32), k, v, 0.25)
    for h in range(4):
        np.testing.assert_allclose(out[h], v[:, h // 2].astype(np.float64).mean(0), atol=1e-13)
    k_same = np.broadcast_to(k[:1], k.shape).copy()
    out = oa.attend_one(_rand(rng, 4, 16), k_same, v, 0.25)
    for h in range(4):
        np.testing.assert_allclose(out[h], v[:, h // 2].astype(np.float64).mean(0), atol=1e-13)


def test_constant_values_pass_through_and_convexity():
    rng = np.random.default_rng(5)
    q, k, v = _rand(rng, 4, 16), _rand(rng, 50, 2, 16), _rand(rng, 50, 2, 16)
    c = _rand(rng, 2, 16)
    out = oa.attend_one(q, k, np.broadcast_to(c[None], (50, 2, 16)).copy(), 0.25)
    for h in range(4):
        np.testing.assert_allclose(out[h], c[h // 2], atol=1e-13)
    out, p = oa.attend_one(q, k, v, 0.25, return_weights=True)
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-12)
    assert (p >= 0).all()
    for h in range(4):
        assert (out[h] <= v[:, h // 2].max(0) + 1e-12).all()
        assert (out[h] >= v[:, h // 2].min(0) - 1e-12).all()


def test_dominant_key_selects_its_value():
    rng = np.random.default_rng(6)
    q = _rand(rng, 2, 16)
    k, v = 0.01 * _rand(rng, 20, 1, 16), _rand(rng, 20, 1, 16)
    k[7, 0] = 50.0 * q[0] / np.linalg.norm(q[0])      # score of token 7 for head 0 >> others
    out = oa.attend_one(q, k, v, 1.0)
    np.testing.assert_allclose(out[0], v[7, 0], atol=1e-9)


def test_scale_and_gqa_mapping_are_not_interchangeable():
    """A wrong head->group map (h % Hkv) or a missing scale must change the answer."""
    rng = np.random.default_rng(7)
    q, k, v = _rand(rng, 6, 8), _rand(rng, 9, 3, 8), _rand(rng, 9, 3, 8)
    out = oa.attend_one(q, k, v, 0.5)
    # head 1 belongs to group 0 (consecutive heads share a KV head): compare with a 1-group call
    solo = oa.attend_one(q[1:2], k[:, 0:1], v[:, 0:1], 0.5)
    np.testing.assert_allclose(out[1], solo[0], atol=1e-14)
    wrong = oa.attend_one(q[1:2], k[:, 1:2], v[:, 1:2], 0.5)
    assert np.abs(out[1] - wrong[0]).max() > 1e-3
    assert np.abs(out - oa.attend_one(q, k, v, 1.0)).max() > 1e-3


# ---- P4: structural invariants -----------------------------------------------------

def _make_layouts(rng, lens, n_kv, d, page=16):
    """Same logical K/V laid out as contiguous slabs, paged blocks and dense padding."""
    caps = [(x + page - 1) // page * page for x in lens]
    n_blocks = sum(caps) // page + 5
    pool_tokens = n_blocks * page
    kc = _rand(rng, pool_tokens, n_kv, d); vc = _rand(rng, pool_tokens, n_kv, d)   # garbage elsewhere
    kp = _rand(rng, pool_tokens, n_kv, d); vp = _rand(rng, pool_tokens, n_kv, d)
    lmax = max(lens)
    kd = _rand(rng, len(lens), lmax, n_kv, d); vd = _rand(rng, len(lens), lmax, n_kv, d)
    bt = wl.shuffled_block_table(np.array(lens), n_blocks, page, seed=9)
    offs, pos = [], 0
    order = rng.permutation(len(lens))          # slabs not in request order
    off_of = {}
    for r in order:
        off_of[r] = pos; pos += caps[r]
    for r, n in enumerate(lens):
        k, v = _rand(rng, n, n_kv, d), _rand(rng, n, n_kv, d)
        offs.append(off_of[r])
        kc[off_of[r]:off_of[r] + n] = k; vc[off_of[r]:off_of[r] + n] = v
        kd[r, :n] = k; vd[r, :n] = v
        for t in range(n):
            row = bt[r, t // page] * page + t % page
            kp[row] = k[t]; vp[row] = v[t]
    return (kc, vc, offs), (kp, vp, bt), (kd, vd)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_layout_independence_is_bit_exact(dtype):
    rng = np.random.default_rng(8)
    lens = [1, 16, 17, 40, 95]
    (kc, vc, offs), (kp, vp, bt), (kd, vd) = _make_layouts(rng, lens, 2, 32)
    q = _rand(rng, len(lens), 6, 32)
    a = oa.decode_attention(q, kc, vc, lens, offsets=offs, dtype=dtype)
    b = oa.decode_attention(q, kp, vp, lens, block_table=bt, dtype=dtype)
    c = oa.decode_attention(q, kd, vd, lens, dense=True, dtype=dtype)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a, c)
    # and it equals the per-request definition on the raw rows
    for r, n in enumerate(lens):
        np.testing.assert_array_equal(a[r], oa.attend_one(q[r], kd[r, :n], vd[r, :n], 1 / math.sqrt(32), dtype))


def test_joint_row_permutation_and_identical_group_queries():
    rng = np.random.default_rng(10)
    k, v = _rand(rng, 64, 2, 16), _rand(rng, 64, 2, 16)
    q = _rand(rng, 6, 16)
    q[1] = q[0]; q[2] = q[0]                    # three heads of group 0 share a query
    out = oa.attend_one(q, k, v, 0.3)
    np.testing.assert_array_equal(out[0], out[1]); np.testing.assert_array_equal(out[0], out[2])
    perm = rng.permutation(64)
    np.testing.assert_allclose(oa.attend_one(q, k[perm], v[perm], 0.3), out, atol=1e-13)


@pytest.mark.parametrize("cuts", [[], [1], [13, 14], [5, 20, 33, 60], list(range(1, 64))])
def test_split_merge_identity(cuts):
    rng = np.random.default_rng(11)
    k, v = 3.0 * _rand(rng, 64, 1, 16), _rand(rng, 64, 1, 16)
    q = _rand(rng, 1, 16)
    full = oa.attend_one(q, k, v, 0.7)[0]
    edges = [0] + cuts + [64]
    parts = [oa.partial_state(q[0], k[a:b, 0], v[a:b, 0], 0.7) for a, b in zip(edges[:-1], edges[1:])]
    merged = oa.merge_splits([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts])
    np.testing.assert_allclose(merged, full, atol=1e-13)
    # a wrong merge (ignoring the max shift) must be caught by this data
    naive = sum(p[2] for p in parts) / sum(p[1] for p in parts)
    if cuts:
        assert np.abs(naive - full).max() > 1e-6


def test_very_negative_score_token_changes_nothing():
    rng = np.random.default_rng(12)
    q, k, v = _rand(rng, 2, 16), _rand(rng, 30, 1, 16), _rand(rng, 30, 1, 16)
    base = oa.attend_one(q, k, v, 1.0)
    # one extra key anti-aligned with both queries' span: score ~ -1e4 for each head
    extra_k = np.zeros((1, 1, 16), np.float32)
    a = np.linalg.lstsq(q.astype(np.float64), -1e4 * np.ones(2), rcond=None)[0]
    extra_k[0, 0] = a.astype(np.float32)
    k2 = np.concatenate([k, extra_k]); v2 = np.concatenate([v, 100 * _rand(rng, 1, 1, 16)])
    np.testing.assert_allclose(oa.attend_one(q, k2, v2, 1.0), base, atol=1e-12)


def test_empty_request_is_zero():
    q = np.ones((2, 8), np.float32)
    out = oa.attend_one(q, np.zeros((0, 1, 8), np.float32), np.zeros((0, 1, 8), np.float32), 1.0)
    assert out.shape == (2, 8) and (out == 0).all()


# ---- P6: bf16 rounding -------------------------------------------------------------

def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(13)
    x = np.concatenate([
        rng.standard_normal(1_000_000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 1_000_000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, -3.3895314e38, np.inf, -np.inf,
                  1e-40, -1e-45, 9.18355e-41, 65280.0, 65408.0], dtype=np.float32),
        # exact ties: mantissa low half == 0x8000 with even / odd upper bit
        np.array([0x3F808000, 0x3F818000, 0x7F7F8000, 0x00008000, 0x00018000], dtype=np.uint32).view(np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16)
    ref_bits = ref.view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(x), ref_bits)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(ref_bits), ref.float().numpy())
    np.testing.assert_array_equal(oa.round_to_bf16(x), ref.float().numpy())
    np.testing.assert_array_equal(oa.widen(ref_bits), ref.float().numpy())


def test_bf16_storage_is_widened_exactly():
    w = wl.qwen_b64()
    k, v = wl.request_kv(w, 0, 3, n_tokens=33)
    q = wl.queries(w, 0)[3]
    assert k.dtype == np.uint16 and q.dtype == np.uint16
    got = oa.attend_one(q, k, v, 1 / math.sqrt(128))
    ref = oa.attend_one(wl.bf16_bits_to_f32(q), wl.bf16_bits_to_f32(k), wl.bf16_bits_to_f32(v), 1 / math.sqrt(128))
    np.testing.assert_array_equal(got, ref)


# ---- workload generator pins (sizes quoted for the seeded configs) -----------------

def test_seeded_workload_sizes():
    assert int(wl.qwen_b64().lengths.sum()) == 46587
    w3 = wl.qwen_b256_pareto()
    assert int(w3.lengths.sum()) == 104745 and int(w3.lengths.max()) == 32768
    assert int(wl.qwen_b128_step().lengths.sum()) == 186585


# ---- FP8 E4M3 storage ------------------------------------------------------------------------

def test_e4m3_decode_table_against_format_definition_and_torch():
    """The oracle's E4M3 widening: values the format fixes, then all 256 codes against torch.float8_e4m3fn."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    got = oa.widen(codes)
    fixed = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0,
             0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0}
    for code, val in fixed.items():
        assert got[code] == np.float32(val), hex(code)
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isfinite(np.delete(got, [0x7F, 0xFF])).all()
    ref = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).float().numpy()
    np.testing.assert_array_equal(np.delete(got, [0x7F, 0xFF]), np.delete(ref, [0x7F, 0xFF]))
    assert (np.diff(got[:0x7F]) > 0).all()                    # positive codes are strictly increasing


def test_e4m3_input_quantiser_rounds_to_nearest_even_and_saturates():
    """workloads.f32_to_e4m3_bits (input generation only): ties, subnormals, saturation; bulk against torch."""
    import torch
    cases = {1.0625: 0x38, 1.1875: 0x3A, 1.3125: 0x3A, 1.4375: 0x3C, 0.001: 0x01, 0.0029: 0x01, 0.0030: 0x02,
             2.0 ** -10: 0x00, 3 * 2.0 ** -10: 0x02, 460.0: 0x7E, 500.0: 0x7E, -1e9: 0xFE, 17.0: 0x58, 0.0: 0x00}
    for x, code in cases.items():
        assert wl.f32_to_e4m3_bits(np.array([x], np.float32))[0] == code, x
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 40
    ref = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(wl.f32_to_e4m3_bits(x), ref)
    np.testing.assert_array_equal(oa.widen(wl.f32_to_e4m3_bits(x)), wl.e4m3_bits_to_f32(wl.f32_to_e4m3_bits(x)))
    err = np.abs(oa.widen(wl.f32_to_e4m3_bits(x)) - np.clip(x, -448, 448))
    assert (err <= np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10)).all()      # half a unit in the last place


def test_fp8_attention_is_attention_over_the_dequantised_values():
    """attend_one takes storage arrays: uint8 K/V are widened through the E4M3 table, nothing else changes."""
    rng = np.random.default_rng(5)
    k8 = wl.f32_to_e4m3_bits(rng.standard_normal((40, 2, 32)).astype(np.float32) * 4)
    v8 = wl.f32_to_e4m3_bits(rng.standard_normal((40, 2, 32)).astype(np.float32) * 4)
    q = wl.f32_to_bf16_bits(rng.standard_normal((4, 32)).astype(np.float32))
    a = oa.attend_one(q, k8, v8, 0.17)
    b = oa.attend_one(q, oa.widen(k8), oa.widen(v8), 0.17)
    np.testing.assert_array_equal(a, b)


# ---- prefill: causal attention of the last n_q tokens (attend_chunk) ------------------------------

def brute_force_chunk(q, k, v, scale):
    """Scalar loops in Python floats: q [n_new][Hq][D], k/v [T][Hkv][D]; query j sees tokens 0 .. T - n_new + j."""
    n_new, n_t = len(q), len(k)
    return np.array([brute_force(q[j], k[:n_t - n_new + j + 1], v[:n_t - n_new + j + 1], scale) for j in range(n_new)])


@pytest.mark.parametrize("seed,n_kv,group,d,n_t,n_new", [(0, 1, 1, 4, 5, 5), (1, 2, 2, 8, 9, 4), (2, 1, 3, 4, 7, 1),
                                                        (3, 2, 1, 4, 6, 6), (4, 1, 7, 8, 12, 5)])
def test_chunk_matches_brute_force(seed, n_kv, group, d, n_t, n_new):
    rng = np.random.default_rng(100 + seed)
    q, k, v = _rand(rng, n_new, n_kv * group, d), _rand(rng, n_t, n_kv, d), _rand(rng, n_t, n_kv, d)
    ref = brute_force_chunk(q.tolist(), k.tolist(), v.tolist(), 0.37)
    np.testing.assert_allclose(oa.attend_chunk(q, k, v, 0.37), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed,n_kv,group,d,n_t,n_new", [(0, 2, 2, 32, 40, 40), (1, 4, 7, 128, 97, 33), (2, 1, 4, 64, 130, 1),
                                                        (3, 2, 8, 128, 64, 64)])
def test_chunk_matches_torch_sdpa_with_causal_mask(seed, n_kv, group, d, n_t, n_new):
    """torch's scaled_dot_product_attention: is_causal for a whole prompt, an explicit lower-right mask for a chunk."""
    rng = np.random.default_rng(200 + seed)
    q, k, v = _rand(rng, n_new, n_kv * group, d), _rand(rng, n_t, n_kv, d), _rand(rng, n_t, n_kv, d)
    scale = 1.0 / math.sqrt(d)
    tq = torch.from_numpy(q).double().permute(1, 0, 2)[None]                              # [1, Hq, n_new, D]
    tk = torch.from_numpy(k).double().permute(1, 0, 2).repeat_interleave(group, 0)[None]  # [1, Hq, T, D]
    tv = torch.from_numpy(v).double().permute(1, 0, 2).repeat_interleave(group, 0)[None]
    if n_new == n_t:
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    else:
        mask = torch.ones(n_new, n_t, dtype=torch.bool).tril(diagonal=n_t - n_new)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(oa.attend_chunk(q, k, v, scale), ref, rtol=0, atol=1e-12)


def test_chunk_rows_are_decode_attention_on_the_prefix():
    """Row j is one decode query over the first len - n_new + j + 1 tokens; bf16 storage goes through the same widening;
    the first token of a fresh prompt returns its own value row; later tokens never influence earlier rows."""
    rng = np.random.default_rng(7)
    n_t, n_new = 75, 30
    q = wl.f32_to_bf16_bits(_rand(rng, n_new, 8, 32))
    k, v = wl.f32_to_bf16_bits(_rand(rng, n_t, 2, 32)), wl.f32_to_bf16_bits(_rand(rng, n_t, 2, 32))
    out = oa.attend_chunk(q, k, v, 0.2)
    for j in range(n_new):
        end = n_t - n_new + j + 1
        np.testing.assert_allclose(out[j], oa.attend_one(q[j], k[:end], v[:end], 0.2), rtol=0, atol=1e-13)
    whole = oa.attend_chunk(q, k[:n_new], v[:n_new], 0.2)
    for h in range(8):
        np.testing.assert_array_equal(whole[0, h], wl.bf16_bits_to_f32(v[0, h // 4]).astype(np.float64))
    k2, v2 = k.copy(), v.copy()
    k2[-1], v2[-1] = wl.f32_to_bf16_bits(_rand(rng, 2, 32)), wl.f32_to_bf16_bits(_rand(rng, 2, 32))
    np.testing.assert_array_equal(oa.attend_chunk(q, k2, v2, 0.2)[:-1], out[:-1])
    assert not np.array_equal(oa.attend_chunk(q, k2, v2, 0.2)[-1], out[-1])
    assert oa.attend_chunk(q[:0], k, v, 0.2).shape == (0, 8, 32)
    with pytest.raises(ValueError):
        oa.attend_chunk(q, k[:10], v[:10], 0.2)
