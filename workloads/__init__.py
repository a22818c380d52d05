"""Seeded synthetic inputs for the ODMA decode hot path.

This module only *draws* inputs (request lengths, predictor outputs, Q/K/V
values, block-table permutations) and rounds them to the storage dtype.  It
holds none of the method's arithmetic: no attention, no softmax, no bucket
assignment, no allocation.  Both the CPU oracle's tests and the GPU path's
tests/benchmarks take their inputs from here, so the two sides see identical
bits.

The paper evaluates on Alpaca and Google-NQ with a trained length predictor
(Section V); neither the datasets nor the predictor are available, so the
distributions below stand in for them: heavy-tailed, high-variance generation
lengths (Section I-A) that drift over time (Section III-C).

All generators use ``numpy.random.default_rng(seed)`` (PCG64).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Optional

import numpy as np

# ----------------------------------------------------------------------------
# storage-dtype rounding (input preparation only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns.

    NaNs are quieted; +-inf and zeros pass through.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    if nan.any():
        rounded = np.where(nan, (bits >> np.uint32(16)) | np.uint32(0x0040), rounded)
    return rounded.astype(np.uint16)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to OCP FP8 E4M3 (1-4-3, bias 7, no infinities; ties to even), as uint8 bit patterns.

    Magnitudes above 448 saturate to 448; NaN becomes 0x7f.  Subnormals (multiples of 2^-9) are kept.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = (x.view(np.uint32) >> np.uint32(24)).astype(np.uint8) & np.uint8(0x80)
    a = np.minimum(np.abs(x).astype(np.float64), 448.0)
    # spacing of representable values around a: 2^(e-3) with e = floor(log2 a) clamped to the subnormal exponent -6
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))
    step = 2.0 ** (e - 3)
    q = np.rint(a / step) * step                       # np.rint rounds half to even; a/step is exact in fp64
    e2 = np.floor(np.log2(np.maximum(q, 2.0 ** -6)))   # rounding may have carried into the next binade
    mant = np.where(q < 2.0 ** -6, q / 2.0 ** -9, (q / 2.0 ** e2 - 1.0) * 8.0)
    expo = np.where(q < 2.0 ** -6, 0.0, e2 + 7.0)
    bits = (expo.astype(np.uint8) << np.uint8(3)) | mant.astype(np.uint8)
    bits = np.where(np.isnan(x), np.uint8(0x7F), bits | sign)
    return bits.astype(np.uint8)


def e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen E4M3 bit patterns (uint8) to fp32 exactly (0x7f and 0xff are NaN)."""
    b = np.asarray(b, dtype=np.uint8)
    e = ((b >> np.uint8(3)) & np.uint8(15)).astype(np.int32)
    m = (b & np.uint8(7)).astype(np.float32)
    mag = np.where(e == 0, m * np.float32(2.0 ** -9), (1.0 + m / 8.0) * np.exp2(e - 7).astype(np.float32))
    mag = np.where((e == 15) & (m == 7), np.float32(np.nan), mag)
    return np.where(b & np.uint8(0x80), -mag, mag).astype(np.float32)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# length distributions
# ----------------------------------------------------------------------------

def lognorm(rng: np.random.Generator, n: int, med: float, sig: float, lo: int, hi: int) -> np.ndarray:
    """Log-normal lengths with the given median, clipped to [lo, hi]."""
    v = np.exp(np.log(med) + sig * rng.standard_normal(n))
    return np.clip(np.rint(v), lo, hi).astype(np.int64)


def pareto(rng: np.random.Generator, n: int, a: float, xm: int, hi: int) -> np.ndarray:
    """Pareto(alpha=a, minimum=xm) lengths, clipped to [xm, hi]."""
    v = xm * (1.0 - rng.random(n)) ** (-1.0 / a)
    return np.clip(np.floor(v), xm, hi).astype(np.int64)


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    """Shapes, allocator geometry and request lengths of one configuration."""
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str                     # "f32" | "bf16" | "fp8" (E4M3 K and V, bf16 queries)
    lengths: np.ndarray               # int64[R], tokens held before decode starts
    boundaries: tuple                 # bucket boundaries b_1 < ... < b_B (tokens)
    main_tokens: int
    safety_tokens: int
    large_cap: int
    data_seed: int
    data_scale: float                 # Q/K/V ~ N(0,1) * data_scale
    align_tokens: int = 16
    page_tokens: int = 16
    extra: dict = field(default_factory=dict)

    @property
    def n_requests(self) -> int:
        return int(self.lengths.shape[0])

    @property
    def pool_tokens(self) -> int:
        return self.main_tokens + self.safety_tokens

    @property
    def kv_bytes_per_token(self) -> int:
        e = {"bf16": 2, "fp8": 1}.get(self.kv_dtype, 4)
        return 2 * self.n_kv_heads * self.head_dim * e


def _round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def tiny(seed: int = 1) -> Workload:
    """Config 1: 1 layer, 4 requests, 2 query heads / 1 KV head, head_dim 64, fp32."""
    lens = np.random.default_rng(seed).integers(16, 129, 4).astype(np.int64)
    return Workload("tiny", 1, 2, 1, 64, "f32", lens, (64, 128, 256),
                    main_tokens=1024, safety_tokens=256, large_cap=256,
                    data_seed=100 + seed, data_scale=1.0)


def qwen_b64(seed: int = 2) -> Workload:
    """Config 2: Qwen2-7B attention shape, batch 64, log-normal context lengths."""
    lens = lognorm(np.random.default_rng(seed), 64, 512, 0.8, 1, 4096)
    return Workload("qwen7b_b64_lognormal", 1, 28, 4, 128, "bf16", lens, (1024, 2048, 4096),
                    main_tokens=64 * 4096, safety_tokens=8 * 4096, large_cap=4096,
                    data_seed=100 + seed, data_scale=1.0 / np.sqrt(128.0))


def qwen_b256_pareto(seed: int = 3, n_layers: int = 1) -> Workload:
    """Config 3: same shape, batch 256, Pareto(1.5, min 128, clip 32768) lengths.

    Bucket boundaries are left to the caller (recalibration on the batch itself);
    ``boundaries`` here is only the initial guess used before recalibration.
    """
    lens = pareto(np.random.default_rng(seed), 256, 1.5, 128, 32768)
    total = int(sum(_round_up(int(x), 16) for x in lens))
    return Workload("qwen7b_b256_pareto", n_layers, 28, 4, 128, "bf16", lens,
                    (256, 512, 2048, 32768),
                    main_tokens=_round_up(2 * total, 4096), safety_tokens=4 * 32768, large_cap=32768,
                    data_seed=100 + seed, data_scale=1.0 / np.sqrt(128.0),
                    extra={"page_seed": 30 + seed})


def qwen_b128_step(seed: int = 4, n_layers: int = 28, steps: int = 64, n_overflow: int = 6) -> Workload:
    """Config 4: 28-layer decode step, batch 128, log-normal (median 1024, clip 8192).

    ``extra`` holds the seeded overflow set: for each chosen request r a step
    k_r in [1, steps) after which its next append overflows its bucket; the
    request starts with ``cap_r - k_r`` tokens.  Everyone else is predicted
    perfectly (its slab holds len0 + steps tokens).
    """
    rng = np.random.default_rng(seed)
    lens = lognorm(rng, 128, 1024, 0.8, 1, 8192 - steps)
    rng2 = np.random.default_rng(40 + seed)
    chosen = np.sort(rng2.choice(128, n_overflow, replace=False))
    k = rng2.integers(1, steps, size=n_overflow)
    return Workload("qwen7b_b128_28layer_step", n_layers, 28, 4, 128, "bf16", lens,
                    (1024, 2048, 4096, 8192),
                    main_tokens=128 * 8192, safety_tokens=16 * 16384, large_cap=16384,
                    data_seed=100 + seed, data_scale=1.0 / np.sqrt(128.0),
                    extra={"steps": steps, "overflow_req": chosen, "overflow_after": k})


# ----------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------

FP8_SCALE = 2.0 ** -6     # de-quantisation factor of the synthetic fp8 pools (values of N(0,1)/sqrt(128) land mid-range)


def draw_values(rng: np.random.Generator, shape, scale: float, kv_dtype: str):
    """N(0,1)*scale values in the storage dtype.

    Returns ``(stored, f32)``: ``stored`` is float32 for "f32", uint16 bf16 bit patterns for
    "bf16", uint8 E4M3 bit patterns (of value / FP8_SCALE) for "fp8"; ``f32`` is the exact fp32
    value of what is stored.
    """
    x = (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    if kv_dtype == "f32":
        return x, x
    if kv_dtype == "fp8":
        # stored value = x / FP8_SCALE rounded to E4M3; the pool's k_scale / v_scale is FP8_SCALE
        b = f32_to_e4m3_bits(x / np.float32(FP8_SCALE))
        return b, e4m3_bits_to_f32(b) * np.float32(FP8_SCALE)
    b = f32_to_bf16_bits(x)
    return b, bf16_bits_to_f32(b)


def request_kv(w: Workload, layer: int, r: int, n_tokens: Optional[int] = None, sharp: bool = False):
    """K and V of request ``r`` in layer ``layer``: two arrays [n_tokens, Hkv, D].

    Each (layer, request) has its own counter-derived seed so requests can be
    generated independently and in any order.  ``sharp`` drops the data scale
    (scores get std ~ sqrt(D)*scale^-1 larger), giving a peaked softmax.
    """
    n = int(w.lengths[r]) if n_tokens is None else int(n_tokens)
    rng = np.random.default_rng([w.data_seed, layer, r, 7])
    scale = 1.0 if sharp else w.data_scale
    k, _ = draw_values(rng, (n, w.n_kv_heads, w.head_dim), scale, w.kv_dtype)
    v, _ = draw_values(rng, (n, w.n_kv_heads, w.head_dim), w.data_scale, w.kv_dtype)
    return k, v


def queries(w: Workload, layer: int, step: int = 0, sharp: bool = False):
    """Decode queries [R, Hq, D] for one layer and step, in the storage dtype."""
    rng = np.random.default_rng([w.data_seed, layer, step, 11])
    scale = 1.0 if sharp else w.data_scale
    q, _ = draw_values(rng, (w.n_requests, w.n_q_heads, w.head_dim), scale, "bf16" if w.kv_dtype == "fp8" else w.kv_dtype)
    return q


def new_token_kv(w: Workload, layer: int, step: int):
    """K and V rows [R, Hkv, D] appended at decode step ``step`` (config 4)."""
    rng = np.random.default_rng([w.data_seed, layer, step, 13])
    k, _ = draw_values(rng, (w.n_requests, w.n_kv_heads, w.head_dim), w.data_scale, w.kv_dtype)
    v, _ = draw_values(rng, (w.n_requests, w.n_kv_heads, w.head_dim), w.data_scale, w.kv_dtype)
    return k, v


def shuffled_block_table(lengths: np.ndarray, n_blocks_total: int, page_tokens: int, seed: int,
                         max_blocks: Optional[int] = None) -> np.ndarray:
    """Paged layout: logical block j of request r lives in physical block bt[r, j].

    Physical ids are a seeded permutation of range(n_blocks_total) dealt out in
    request order; unused entries are -1.
    """
    need = [(int(x) + page_tokens - 1) // page_tokens for x in lengths]
    if sum(need) > n_blocks_total:
        raise ValueError("paged pool too small")
    mb = max(need) if max_blocks is None else max_blocks
    perm = np.random.default_rng(seed).permutation(n_blocks_total).astype(np.int32)
    bt = np.full((len(need), mb), -1, dtype=np.int32)
    pos = 0
    for r, nb in enumerate(need):
        bt[r, :nb] = perm[pos:pos + nb]
        pos += nb
    return bt


# ----------------------------------------------------------------------------
# config 5: drifting arrival stream with a synthetic predictor
# ----------------------------------------------------------------------------

@dataclass
class Arrival:
    total_len: int       # realized total KV length L at completion
    prefilled: int       # tokens present on admission (L - g)
    decode_steps: int    # g
    pred_len: int        # synthetic predictor's estimate of L
    uncertainty: float   # u in [0, 1]


def drift_arrivals(seed: int = 5, n_steps: int = 1000, lo_median: float = 256.0, sigma: float = 0.8,
                   alpha: float = 1.2, xmin: int = 128, clip: int = 65536) -> Iterator:
    """Generator protocol for the drift run: ``send(step)`` returns one Arrival.

    A request admitted at step s draws its total length from a mixture: with
    probability s/(n_steps-1) Pareto(alpha, xmin) else log-normal(lo_median,
    sigma), both clipped to [2, clip].  The synthetic predictor sees
    L_hat = ceil(L * exp(0.1 z)), u = min(1, |z|/3), z ~ N(0,1).
    """
    rng = np.random.default_rng(seed)
    step = yield None
    while True:
        frac = min(1.0, max(0.0, step / float(max(1, n_steps - 1))))
        if rng.random() < frac:
            L = int(pareto(rng, 1, alpha, xmin, clip)[0])
        else:
            L = int(lognorm(rng, 1, lo_median, sigma, 2, clip)[0])
        g = int(rng.integers(8, 65))
        g = max(1, min(g, L - 1))
        z = float(rng.standard_normal())
        pred = int(np.ceil(L * np.exp(0.1 * z)))
        u = float(min(1.0, abs(z) / 3.0))
        step = yield Arrival(L, L - g, g, pred, u)
