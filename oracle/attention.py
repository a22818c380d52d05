"""Oracle: decode attention over the ODMA KV layouts (test infrastructure only).

ODMA changes *where* a request's KV bytes live (one contiguous slab per request,
Section I-C and III-A of the paper), not what attention computes (the paper keeps
the stock kernels, Section IV-A and VI).  The result therefore has a plain
definition -- scaled dot-product softmax attention of one query per head over
all ``len_r`` cached tokens (Vaswani et al., the paper's reference for the
Transformer) -- and this file is that definition written out with numpy:

    s_t        = sm_scale * sum_d q[r,h,d] * K_r[t,g,d]        g = h // (Hq/Hkv)
    p_t        = exp(s_t - max_t s_t) / sum_t exp(s_t - max_t s_t)
    out[r,h,d] = sum_t p_t * V_r[t,g,d]

The query attends to every cached token including the one appended this step;
there is no mask, bias, rotary step or soft-cap inside the slab.  Inputs arrive
in their storage dtype (fp32 arrays, or uint16 arrays holding bf16 bit
patterns), are widened exactly, and the arithmetic runs in ``dtype`` (float64 by
default, float32 on request).

The three layouts differ only in how the rows of K_r and V_r are *found*:

    contiguous : row t of request r is pool[off_r + t]               (ODMA slab)
    paged      : row t is pool[bt[r, t // P] * P + t % P]            (block table)
    dense      : row t is dense[r, t]                                 (padded)

All three gather the rows into the same [len, Hkv, D] array and then run the
same code, so results are bit-identical across layouts.

``merge_splits`` is the log-sum-exp combination of partial results computed on
disjoint token ranges (the cross-split reduction of a split-K decode); it is
exact up to rounding and is pinned against the one-pass definition.

``attend_chunk`` is the prefill counterpart: the last n_q tokens of a request each carry a
query, and query j (at position len - n_q + j) sees tokens 0 .. len - n_q + j of the same slab
(causal self-attention; a whole prompt is the case n_q = len, a later chunk of a long prompt
has n_q < len).  Row j of its result is by definition ``attend_one`` on the first
len - n_q + j + 1 tokens; the function is written with an explicit visibility mask instead,
and the two are pinned against each other.

Pins (tests/test_oracle_attention.py): brute-force scalar loops in Python
floats; ``torch.nn.functional.scaled_dot_product_attention`` on CPU; closed forms
(len = 1, zero query, constant V, one dominant key); convexity bounds; layout
independence; split-merge identity; bf16 rounding against torch.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


# ---------------------------------------------------------------------------
# storage dtypes
# ---------------------------------------------------------------------------

def widen(x: np.ndarray) -> np.ndarray:
    """Storage array -> float32 values, exactly.  uint16 means bf16 bit patterns."""
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if x.dtype == np.float32:
        return x
    if x.dtype == np.uint8:
        return _E4M3[x]
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def _e4m3_table() -> np.ndarray:
    """All 256 values of OCP FP8 E4M3: sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent 0 is
    subnormal (m * 2^-9), there are no infinities, and S.1111.111 is NaN."""
    t = np.zeros(256, dtype=np.float32)
    for code in range(256):
        e, m = (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            v = float("nan")
        elif e == 0:
            v = m * 2.0 ** -9
        else:
            v = (8 + m) * 2.0 ** (e - 10)
        t[code] = -v if code & 0x80 else v
    return t


_E4M3 = _e4m3_table()


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Values -> nearest bf16 (ties to even), returned as float32 values."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    bits = x32.view(np.uint32)
    keep = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return keep.view(np.float32)


# ---------------------------------------------------------------------------
# layouts: index mapping only
# ---------------------------------------------------------------------------

def rows_contiguous(pool: np.ndarray, offset: int, length: int) -> np.ndarray:
    """Rows [offset, offset+length) of a token-major pool [pool_tokens, Hkv, D]."""
    if offset < 0 or offset + length > pool.shape[0]:
        raise IndexError("slab outside the pool")
    return pool[offset:offset + length]


def rows_paged(pool: np.ndarray, block_row: np.ndarray, length: int, page_tokens: int) -> np.ndarray:
    """Rows of a request whose logical block j is physical block block_row[j]."""
    t = np.arange(length, dtype=np.int64)
    blk = block_row[t // page_tokens].astype(np.int64)
    if length and (blk.min() < 0 or (blk.max() + 1) * page_tokens > pool.shape[0]):
        raise IndexError("block table points outside the pool")
    return pool[blk * page_tokens + t % page_tokens]


def rows_dense(dense: np.ndarray, r: int, length: int) -> np.ndarray:
    """Rows [0, length) of request r in a padded dense tensor [R, Lmax, Hkv, D]."""
    return dense[r, :length]


# ---------------------------------------------------------------------------
# the definition
# ---------------------------------------------------------------------------

def attend_one(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float, dtype=np.float64,
               return_weights: bool = False):
    """One request: q [Hq, D], k and v [len, Hkv, D] (storage dtype) -> out [Hq, D].

    A request with len == 0 has an empty softmax; its output is defined as 0.
    """
    qf = widen(q).astype(dtype)
    kf = widen(k).astype(dtype)
    vf = widen(v).astype(dtype)
    n_q, d = qf.shape
    n_tok, n_kv, _ = kf.shape
    if n_q % n_kv:
        raise ValueError("query heads must be a multiple of KV heads")
    group = n_q // n_kv
    out = np.zeros((n_q, d), dtype=dtype)
    weights = np.zeros((n_q, n_tok), dtype=dtype)
    if n_tok == 0:
        return (out, weights) if return_weights else out
    scale = dtype(sm_scale)
    for h in range(n_q):
        g = h // group
        s = (kf[:, g, :] @ qf[h]) * scale              # [len]
        e = np.exp(s - s.max())
        p = e / e.sum()
        out[h] = p @ vf[:, g, :]
        weights[h] = p
    return (out, weights) if return_weights else out


def attend_chunk(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float, dtype=np.float64) -> np.ndarray:
    """Causal attention of the last n_q tokens of one request: q [n_q, Hq, D], k and v [len, Hkv, D]
    (storage dtype, len >= n_q) -> out [n_q, Hq, D].  Query j sits at position len - n_q + j and sees
    tokens 0 .. len - n_q + j."""
    qf = widen(q).astype(dtype)
    kf = widen(k).astype(dtype)
    vf = widen(v).astype(dtype)
    n_new, n_q, d = qf.shape
    n_tok, n_kv, _ = kf.shape
    if n_new > n_tok:
        raise ValueError("more query tokens than cached tokens")
    if n_q % n_kv:
        raise ValueError("query heads must be a multiple of KV heads")
    group = n_q // n_kv
    out = np.zeros((n_new, n_q, d), dtype=dtype)
    if n_new == 0:
        return out
    position = n_tok - n_new + np.arange(n_new)
    visible = np.arange(n_tok)[None, :] <= position[:, None]          # [n_new, len]
    scale = dtype(sm_scale)
    for h in range(n_q):
        g = h // group
        s = (qf[:, h, :] @ kf[:, g, :].T) * scale                    # [n_new, len]
        s = np.where(visible, s, -np.inf)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vf[:, g, :]
    return out


def decode_attention(q: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray,
                     lengths: Sequence[int], *, offsets: Optional[Sequence[int]] = None,
                     block_table: Optional[np.ndarray] = None, page_tokens: int = 16,
                     dense: bool = False, sm_scale: Optional[float] = None,
                     dtype=np.float64, out_bf16: bool = False) -> np.ndarray:
    """Batched decode attention, q [R, Hq, D] -> out [R, Hq, D] in ``dtype``.

    Exactly one layout applies: ``offsets`` (contiguous slabs in pools
    [pool_tokens, Hkv, D]), ``block_table`` (paged, same pool shape) or
    ``dense=True`` (k_pool, v_pool are [R, Lmax, Hkv, D]).  ``out_bf16`` rounds
    the result to bf16 values (still returned in ``dtype``).
    """
    n_layouts = (offsets is not None) + (block_table is not None) + bool(dense)
    if n_layouts != 1:
        raise ValueError("choose exactly one layout")
    n_req, n_q, d = q.shape
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(float(d))
    out = np.zeros((n_req, n_q, d), dtype=dtype)
    for r in range(n_req):
        n = int(lengths[r])
        if offsets is not None:
            k = rows_contiguous(k_pool, int(offsets[r]), n)
            v = rows_contiguous(v_pool, int(offsets[r]), n)
        elif block_table is not None:
            k = rows_paged(k_pool, block_table[r], n, page_tokens)
            v = rows_paged(v_pool, block_table[r], n, page_tokens)
        else:
            k = rows_dense(k_pool, r, n)
            v = rows_dense(v_pool, r, n)
        out[r] = attend_one(q[r], k, v, sm_scale, dtype)
    if out_bf16:
        out = round_to_bf16(out).astype(dtype)
    return out


# ---------------------------------------------------------------------------
# cross-split reduction
# ---------------------------------------------------------------------------

def partial_state(q_h: np.ndarray, k_g: np.ndarray, v_g: np.ndarray, sm_scale: float, dtype=np.float64):
    """Un-normalised softmax state of one head on one token range.

    Returns (m, l, o): m = max score, l = sum exp(s - m), o[d] = sum exp(s - m) v[t, d].
    """
    s = (widen(k_g).astype(dtype) @ widen(q_h).astype(dtype)) * dtype(sm_scale)
    m = s.max()
    e = np.exp(s - m)
    return m, e.sum(), e @ widen(v_g).astype(dtype)


def merge_splits(ms: Sequence[float], ls: Sequence[float], os: Sequence[np.ndarray]) -> np.ndarray:
    """Combine per-range (m_i, l_i, o_i): m* = max m_i, w_i = exp(m_i - m*),
    out = sum w_i o_i / sum w_i l_i."""
    ms = np.asarray(ms)
    m_star = ms.max()
    w = np.exp(ms - m_star)
    l_star = (w * np.asarray(ls)).sum()
    o_star = sum(wi * oi for wi, oi in zip(w, os))
    return o_star / l_star
