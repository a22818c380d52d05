"""Test-side plumbing for the GPU parity tests: device buffers (torch), pool filling
through odma_append_kv, decode calls, and the comparison against the CPU oracle.

The HIP path never sees oracle code and the oracle never sees device results: both
get the same seeded inputs from ``workloads``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

import workloads as wl
from oracle import attention as oa
from paper_2512_09427_amd import binding as B

DEV = "cuda:0"

# spec tolerance for bf16-in / fp32-accumulate attention
ABS_TOL, REL_TOL = 2e-3, 1e-2


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def storage_dtype(kv_dtype: str):
    return {"bf16": torch.int16, "fp8": torch.uint8}.get(kv_dtype, torch.float32)


@dataclass
class DevicePool:
    pool: B.Pool
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    workspace: torch.Tensor
    w: wl.Workload
    out_dtype: int

    @property
    def out_torch_dtype(self):
        return torch.int16 if self.out_dtype == B.BF16 else torch.float32


def make_pool(w: wl.Workload, *, out_dtype: Optional[int] = None, decode_kernel: int = B.KERNEL_AUTO,
              n_layers: Optional[int] = None, max_requests: Optional[int] = None, poison: bool = True,
              max_splits: int = 0, quantiles=None, window: int = 10000) -> DevicePool:
    kv = {"bf16": B.BF16, "fp8": B.FP8}.get(w.kv_dtype, B.F32)
    out_dtype = (B.BF16 if kv == B.FP8 else kv) if out_dtype is None else out_dtype
    L = w.n_layers if n_layers is None else n_layers
    elems = L * w.n_kv_heads * w.pool_tokens * w.head_dim
    sd = storage_dtype(w.kv_dtype)
    if poison:
        # every slot starts as a NaN bit pattern: a kernel that lets stale slots leak shows up at once
        fill = -1 if sd == torch.int16 else 0x7f if sd == torch.uint8 else float("nan")
        k_pool = torch.full((elems,), fill, dtype=sd, device=DEV)
        v_pool = torch.full((elems,), fill, dtype=sd, device=DEV)
    else:
        k_pool = torch.zeros(elems, dtype=sd, device=DEV)
        v_pool = torch.zeros(elems, dtype=sd, device=DEV)
    nreq = max_requests or max(w.n_requests, 1)
    args = dict(n_layers=L, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, kv_dtype=kv,
                out_dtype=out_dtype, main_tokens=w.main_tokens, safety_tokens=w.safety_tokens, large_cap=w.large_cap,
                boundaries=w.boundaries, max_requests=nreq, align_tokens=w.align_tokens,
                decode_kernel=decode_kernel, max_splits=max_splits, quantiles=quantiles, window=window)
    if kv == B.FP8:
        args.update(k_scale=wl.FP8_SCALE, v_scale=wl.FP8_SCALE)
    cfg0, _ = B.make_config(**args)
    ws = torch.empty(B.odma_workspace_bytes(cfg0), dtype=torch.uint8, device=DEV)
    cfg, keep = B.make_config(**args, k_pool=k_pool, v_pool=v_pool, workspace=ws)
    return DevicePool(B.Pool(cfg, keep), k_pool, v_pool, ws, w, out_dtype)


def fill(dp: DevicePool, layer: int, kv_rows: Sequence, *, offsets: Optional[np.ndarray] = None,
         block_table: Optional[np.ndarray] = None, positions: Optional[np.ndarray] = None):
    """Appends kv_rows[r] = (k, v), each [n_r, Hkv, D] in storage dtype, for every request in one call."""
    n = len(kv_rows)
    counts = np.array([k.shape[0] for k, _ in kv_rows], dtype=np.int32)
    if counts.sum() == 0:
        return
    start = np.concatenate([[0], np.cumsum(counts)[:-1]]).astype(np.int64)
    k_all = np.concatenate([k for k, _ in kv_rows], axis=0)
    v_all = np.concatenate([v for _, v in kv_rows], axis=0)
    pos = np.zeros(n, np.int32) if positions is None else np.asarray(positions, np.int32)
    bt = None if block_table is None else to_dev(block_table.astype(np.int32))
    dp.pool.odma_append_kv(layer, n, None if offsets is None else to_dev(np.asarray(offsets, np.int64)),
                           to_dev(pos), to_dev(counts), to_dev(start), int(counts.max()),
                           bt, 0 if bt is None else block_table.shape[1], to_dev(k_all), to_dev(v_all))
    torch.cuda.synchronize()


def append_one(dp: DevicePool, layer: int, k_new: np.ndarray, v_new: np.ndarray, positions: np.ndarray, *,
               offsets: Optional[np.ndarray] = None, block_table: Optional[np.ndarray] = None):
    """Decode-step append: one row per request."""
    n = k_new.shape[0]
    bt = None if block_table is None else to_dev(block_table.astype(np.int32))
    dp.pool.odma_append_kv(layer, n, None if offsets is None else to_dev(np.asarray(offsets, np.int64)),
                           to_dev(np.asarray(positions, np.int32)), None, None, 1,
                           bt, 0 if bt is None else block_table.shape[1], to_dev(k_new), to_dev(v_new))


def decode(dp: DevicePool, layer: int, q: np.ndarray, lengths: np.ndarray, *, offsets: Optional[np.ndarray] = None,
           block_table: Optional[np.ndarray] = None, flags: int = 0) -> np.ndarray:
    """Runs odma_decode_attention; returns out [n, Hq, D] as float32 values."""
    n = q.shape[0]
    out = torch.full((n, dp.w.n_q_heads, dp.w.head_dim), -1 if dp.out_dtype == B.BF16 else float("nan"),
                     dtype=dp.out_torch_dtype, device=DEV)
    bt = None if block_table is None else to_dev(block_table.astype(np.int32))
    dp.pool.odma_decode_attention(layer, n, to_dev(q), None if offsets is None else to_dev(np.asarray(offsets, np.int64)),
                                  to_dev(np.asarray(lengths, np.int32)), bt,
                                  0 if bt is None else block_table.shape[1], out, flags)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    if dp.out_dtype == B.BF16:
        res = wl.bf16_bits_to_f32(res.view(np.uint16))
    return res


def decode_step(dp: DevicePool, layer: int, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, lengths_after: np.ndarray,
                *, offsets: Optional[np.ndarray] = None, block_table: Optional[np.ndarray] = None, flags: int = 0):
    """Runs odma_decode_step (fused append + attention); returns out [n, Hq, D] as float32 values."""
    n = q.shape[0]
    out = torch.full((n, dp.w.n_q_heads, dp.w.head_dim), -1 if dp.out_dtype == B.BF16 else float("nan"),
                     dtype=dp.out_torch_dtype, device=DEV)
    bt = None if block_table is None else to_dev(block_table.astype(np.int32))
    dp.pool.odma_decode_step(layer, n, to_dev(q), to_dev(k_new), to_dev(v_new),
                             None if offsets is None else to_dev(np.asarray(offsets, np.int64)),
                             to_dev(np.asarray(lengths_after, np.int32)), bt,
                             0 if bt is None else block_table.shape[1], out, flags)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    if dp.out_dtype == B.BF16:
        res = wl.bf16_bits_to_f32(res.view(np.uint16))
    return res


def prefill(dp: DevicePool, layer: int, q_rows: np.ndarray, q_start: np.ndarray, n_q: np.ndarray, lengths: np.ndarray, *,
            offsets: Optional[np.ndarray] = None, block_table: Optional[np.ndarray] = None,
            total_q: Optional[int] = None) -> np.ndarray:
    """Runs odma_prefill_attention; q_rows [total, Hq, D] bf16 bits; returns out [total, Hq, D] as float32 values
    (rows the call does not write keep the NaN pattern they were filled with)."""
    total = q_rows.shape[0]
    out = torch.full((total, dp.w.n_q_heads, dp.w.head_dim), -1 if dp.out_dtype == B.BF16 else float("nan"),
                     dtype=dp.out_torch_dtype, device=DEV)
    bt = None if block_table is None else to_dev(block_table.astype(np.int32))
    dp.pool.odma_prefill_attention(layer, len(n_q), to_dev(q_rows), total if total_q is None else total_q,
                                   to_dev(np.asarray(q_start, np.int64)), to_dev(np.asarray(n_q, np.int32)),
                                   None if offsets is None else to_dev(np.asarray(offsets, np.int64)),
                                   to_dev(np.asarray(lengths, np.int32)), bt, 0 if bt is None else block_table.shape[1], out)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    if dp.out_dtype == B.BF16:
        res = wl.bf16_bits_to_f32(res.view(np.uint16))
    return res


def gather(dp: DevicePool, layer: int, offset: int, length: int, block_row: Optional[np.ndarray] = None):
    sd = storage_dtype(dp.w.kv_dtype)
    k = torch.zeros((length, dp.w.n_kv_heads, dp.w.head_dim), dtype=sd, device=DEV)
    v = torch.zeros_like(k)
    br = None if block_row is None else to_dev(block_row.astype(np.int32))
    dp.pool.odma_gather_kv(layer, offset, length, br, k, v)
    torch.cuda.synchronize()
    k, v = k.cpu().numpy(), v.cpu().numpy()
    if dp.w.kv_dtype == "bf16":
        k, v = k.view(np.uint16), v.view(np.uint16)
    return k, v


def oracle_out(w: wl.Workload, q: np.ndarray, kv_rows: Sequence, dtype=np.float64, out_bf16: bool = False,
               sm_scale: Optional[float] = None) -> np.ndarray:
    scale = 1.0 / math.sqrt(w.head_dim) if sm_scale is None else sm_scale
    if w.kv_dtype == "fp8":
        # stored bytes are value / FP8_SCALE: the K factor joins the softmax scale, the V factor the output
        scale *= wl.FP8_SCALE
    out = np.stack([oa.attend_one(q[r], kv_rows[r][0], kv_rows[r][1], scale, dtype) for r in range(len(kv_rows))])
    if w.kv_dtype == "fp8":
        out = out * dtype(wl.FP8_SCALE)
    if out_bf16:
        out = oa.round_to_bf16(out).astype(dtype)
    return out


def check(got: np.ndarray, ref: np.ndarray, abs_tol: float = ABS_TOL, rel_tol: float = REL_TOL, what: str = ""):
    """|got - ref| <= abs_tol + rel_tol*|ref| elementwise; returns max error / max |ref| for reporting."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got.astype(np.float64) - ref)
    bound = abs_tol + rel_tol * np.abs(ref)
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements out of tolerance; worst at {idx}: "
                             f"got {got[idx]!r} ref {ref[idx]!r} err {err[idx]:.3e}")
    scale = np.abs(ref).max()
    return float(err.max() / scale) if scale > 0 else 0.0


def assign_perfect(dp: DevicePool, lengths: np.ndarray, extra: int = 0):
    """Admits every request with its true length (+extra) as the prediction; returns offsets, caps."""
    n = len(lengths)
    rc, bk, off, cap, st = dp.pool.odma_assign(np.arange(n), (np.asarray(lengths) + extra))
    assert rc == 0, (rc, st)
    return off, cap


# ---------------------------------------------------------------------------------------
# smoke: one tiny invocation of the hot path on cuda:0 against the oracle
# ---------------------------------------------------------------------------------------

def run_smoke():
    assert torch.cuda.is_available(), "smoke() needs a GPU"
    # Tiny configuration (fp32, VALU kernel): assign -> append -> decode, against the oracle
    w = wl.tiny()
    dp = make_pool(w)
    off, _ = assign_perfect(dp, w.lengths)
    kv = [wl.request_kv(w, 0, r) for r in range(w.n_requests)]
    fill(dp, 0, kv, offsets=off)
    q = wl.queries(w, 0)
    got = decode(dp, 0, q, w.lengths, offsets=off)
    rel = check(got, oracle_out(w, q, kv), 1e-5, 1e-5, "tiny")
    print(f"smoke tiny (fp32, VALU kernel): max err / max|ref| = {rel:.2e}")
    # a few Qwen-shaped bf16 requests through the MFMA kernel, one of them split over chunks
    w2 = wl.qwen_b64()
    w2.lengths = np.array([1, 17, 300, 2500, 64, 1023], dtype=np.int64)
    dp2 = make_pool(w2, max_requests=8)
    off2, _ = assign_perfect(dp2, w2.lengths)
    kv2 = [wl.request_kv(w2, 0, r, sharp=True) for r in range(6)]
    fill(dp2, 0, kv2, offsets=off2)
    q2 = wl.queries(w2, 0, sharp=True)
    got2 = decode(dp2, 0, q2, w2.lengths, offsets=off2)
    rel2 = check(got2, oracle_out(w2, q2, kv2), what="qwen-shaped bf16")
    assert dp2.pool.odma_pool_decode_kernel() == B.KERNEL_MFMA
    print(f"smoke qwen-shaped (bf16, MFMA kernel): max err / max|ref| = {rel2:.2e}")
    # the same requests as whole prompts through the prefill kernel (causal attention of every token)
    n_q = w2.lengths
    q_start = np.concatenate([[0], np.cumsum(n_q)[:-1]])
    q_rows, _ = wl.draw_values(np.random.default_rng(3), (int(n_q.sum()), w2.n_q_heads, w2.head_dim), 1.0, "bf16")
    got3 = prefill(dp2, 0, q_rows, q_start, n_q, w2.lengths, offsets=off2)
    ref3 = np.concatenate([oa.attend_chunk(q_rows[s:s + c], kv2[r][0], kv2[r][1], 1.0 / math.sqrt(w2.head_dim))
                           for r, (s, c) in enumerate(zip(q_start, n_q))])
    rel3 = check(got3, ref3, what="prefill")
    print(f"smoke prefill (bf16, whole prompts): max err / max|ref| = {rel3:.2e}")
    # and on fp8 (E4M3) pools
    w4 = wl.qwen_b64()
    w4.kv_dtype = "fp8"
    w4.lengths = np.array([1, 33, 300, 2500], dtype=np.int64)
    dp4 = make_pool(w4, max_requests=8)
    off4, _ = assign_perfect(dp4, w4.lengths)
    kv4 = [wl.request_kv(w4, 0, r, sharp=True) for r in range(4)]
    fill(dp4, 0, kv4, offsets=off4)
    q4 = wl.queries(w4, 0, sharp=True)
    rel4 = check(decode(dp4, 0, q4, w4.lengths, offsets=off4), oracle_out(w4, q4, kv4), what="fp8 pools")
    print(f"smoke fp8 pools (E4M3 K/V, MFMA kernel): max err / max|ref| = {rel4:.2e}")
