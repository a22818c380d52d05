// Prefill (chunk) attention for gfx950: the last n_q tokens of every request each carry a
// query and attend causally to the request's slab (bf16 storage, head_dim 128, G <= 16).
//
// Unlike decode this is a dense contraction with reuse: one 16-token K/V tile serves every
// query column.  The (token, head-in-group) pairs of one (request, KV head) are flattened into
// columns  col = j * G + h  (j: query token of the chunk, h: head inside the GQA group), so any
// group size fills the 16-wide matrix tiles.  A work item is 64 CT consecutive columns of one
// (request, KV head): four waves of a work-group take CT 16-column tiles each, whose Q operands
// and O accumulators stay in registers, and share the K/V tiles the item can see through LDS.
// CT = 4 (256-column items, one work-group per CU) has the most reuse per K/V byte.  CT = 2 halves the
// registers so that two work-groups share a CU and one's LDS reads and item start run under the other's
// matrix instructions: +12 to +25 % on every prompt mix measured, and the default.
//
// Items are handed out through an atomic counter (persistent work-groups, heaviest columns of a
// request first), because causal items differ in length by construction.
#pragma once

#include "kernels_common.h"

namespace {

constexpr int PREFILL_PLAN_THREADS = 256;

struct PrefillHeader {
  int32_t n_items;
  int32_t next_item;       // work queue cursor, reset by the plan kernel
  int32_t avg_pairs;       // mean number of 32-token K/V pairs an item streams (estimate of the plan)
  int32_t pad1;
};

struct PrefillArgs {
  const char* k;             // layer base of the K pool
  const char* v;
  const unsigned short* q;   // [total_q][Hq][128] bf16
  void* out;                 // [total_q][Hq][128]
  const int64_t* q_start;    // [n] first row of request r in q / out
  const int32_t* n_q;        // [n] query tokens of request r (the last n_q of its lengths[r] tokens)
  const int64_t* offsets;    // [n] slab base (tokens) or nullptr when paged
  const int32_t* lengths;    // [n]
  const int32_t* bt;
  int32_t bt_stride;
  PrefillHeader* hdr;
  const int32_t* item_start; // [n + 1] exclusive prefix of items per request
  int32_t n, Hq, Hkv, G;
  int64_t total_q;           // rows of q and out: rows at or past it are never touched
  int64_t head_stride;
  float scale_log2;          // sm_scale * log2(e) (fp8 pools: times k_scale)
  float out_scale;           // 1, or v_scale for fp8 pools
  int32_t out_bf16;
};

// query tokens of request r that are really there: never more than the tokens it holds, never
// past the end of q
__device__ __forceinline__ int prefill_rows(const int32_t* n_q, const int32_t* lengths, const int64_t* q_start,
                                            int64_t total_q, int r) {
  int64_t rows = min(n_q[r], lengths[r]);
  const int64_t s = q_start[r];
  if (s < 0 || rows < 0) return 0;
  rows = min(rows, total_q - s);
  return rows > 0 ? (int)rows : 0;
}

// one work-group: items per request -> exclusive prefix, total, queue cursor
__global__ __launch_bounds__(PREFILL_PLAN_THREADS) void prefill_plan_kernel(const int32_t* __restrict__ n_q,
                                                                           const int32_t* __restrict__ lengths,
                                                                           const int64_t* __restrict__ q_start,
                                                                           int64_t total_q, int32_t n, int32_t Hkv, int32_t G,
                                                                           int32_t cols_item, PrefillHeader* hdr,
                                                                           int32_t* item_start) {
  __shared__ int part[PREFILL_PLAN_THREADS];
  const int tid = threadIdx.x;
  const int per = (n + PREFILL_PLAN_THREADS - 1) / PREFILL_PLAN_THREADS;
  const int r0 = min(tid * per, n), r1 = min(r0 + per, n);
  auto items_of = [&](int r) {
    const int64_t cols = (int64_t)prefill_rows(n_q, lengths, q_start, total_q, r) * G;
    return (int)((cols + cols_item - 1) / cols_item) * Hkv;
  };
  int sum = 0;
  long long work = 0;                                      // pairs streamed by this thread's requests, all items together
  for (int r = r0; r < r1; ++r) {
    const int items = items_of(r);
    sum += items;
    // an item of request r sees on average len - rows / 2 keys
    const int rows = prefill_rows(n_q, lengths, q_start, total_q, r);
    work += (long long)items * ((lengths[r] - rows / 2 + 31) / 32);
  }
  __shared__ long long work_all;
  if (tid == 0) work_all = 0;
  __syncthreads();
  atomicAdd((unsigned long long*)&work_all, (unsigned long long)work);
  part[tid] = sum;
  __syncthreads();
  for (int o = 1; o < PREFILL_PLAN_THREADS; o <<= 1) {
    const int add = tid >= o ? part[tid - o] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int run = part[tid] - sum;
  for (int r = r0; r < r1; ++r) {
    item_start[r] = run;
    run += items_of(r);
  }
  if (tid == PREFILL_PLAN_THREADS - 1) {
    item_start[n] = part[tid];
    hdr->n_items = part[tid];
    hdr->next_item = 0;
    hdr->avg_pairs = (int)(work_all / max(part[tid], 1));
    hdr->pad1 = 0;
  }
}

// LDS stage of one pair of tiles (32 tokens): K of both tiles as loaded (the 16x16x32 A operands of
// S^T = K Q^T), and V rearranged into the A operands of O^T += V^T P^T over the 32 tokens: for channel
// group dt, lane (c, q) finds channels c of tokens 4q .. 4q+3 of the first tile followed by the same of
// the second tile in one 16-byte piece.
constexpr int PREFILL_STAGE_BYTES = 16384;
constexpr int PREFILL_STAGES = 2;

// two E4M3 bytes of a word -> two bf16 bit patterns in one word (exact: E4M3 values are bf16 values)
template <bool HIGH_HALF>
__device__ __forceinline__ unsigned fp8x2_to_bf16x2(unsigned w) {
  typedef float float2v __attribute__((ext_vector_type(2)));
  const float2v f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, HIGH_HALF);
  return (__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u);
}

// FP8: the pools hold E4M3 bytes (2 KiB blocks in the fp8 operand order of the decode kernel); the loader waves
// widen them to bf16 on the way into LDS and store them in the bf16 layout, everything after that is shared.
template <bool PAGED, int CT, bool FP8>
__global__ __launch_bounds__(256, CT == 4 ? 1 : 2) void prefill_kernel(PrefillArgs a) {
  constexpr int TILE_BYTES = BLK * 128 * (FP8 ? 1 : 2);
  constexpr int LOADS = TILE_BYTES / 1024;                         // 16-byte loads per lane and tile
  constexpr int COLS_WAVE = 16 * CT, COLS_ITEM = 4 * COLS_WAVE;     // CT column tiles per wave, four waves per item
  __shared__ __attribute__((aligned(16))) char stage_mem[PREFILL_STAGES * PREFILL_STAGE_BYTES];
  __shared__ int item_slot, redo_slot;
  const int lane = threadIdx.x & 63, wv = rfl(threadIdx.x >> 6);
  const int col16 = lane & 15, g4 = lane >> 4;
  const int G = a.G;
  const float NEG_INF = -INFINITY;
  // loader role of this wave: waves 0, 1 bring the K tiles of a pair, waves 2, 3 the V tiles
  const bool loads_v = wv >= 2;
  const int which = wv & 1;                                            // first or second tile of the pair
  const char* src_base = (loads_v ? a.v : a.k) + lane * 16;

  // Work queue: one counter in memory, which answers about 14 M requests a second on this part -- with
  // thousands of small items that alone would bound the kernel.  A work-group therefore takes a run of
  // consecutive items per request, long enough to stream about 64 K/V pairs (some 40 us) but never more
  // than an eighth of its share of the items, so that large items still balance one by one; and it asks
  // one run ahead: the answer travels while the current run is computed.
  const int n_items = a.hdr->n_items;
  const int run = min(min(max(64 / max(a.hdr->avg_pairs, 1), 1), 16), max(n_items / ((int)gridDim.x * 8), 1));
  int ahead = 0;
  if (threadIdx.x == 0) ahead = atomicAdd(&a.hdr->next_item, run);
  int next = 0, run_end = 0;
  for (;;) {
    // ---- next item (every wave reaches the exit together)
    __syncthreads();                                       // the previous item's slot and stages are done with
    if (next == run_end) {
      if (threadIdx.x == 0) item_slot = ahead;
      __syncthreads();
      next = rfl(item_slot);
      if (next >= n_items) break;
      run_end = min(next + run, n_items);
      if (threadIdx.x == 0) ahead = atomicAdd(&a.hdr->next_item, run);
    }
    const int item = next++;
    // request of the item: largest r with item_start[r] <= item (item_start is non-decreasing; empty
    // requests repeat a value, so take the last one that still has items).  Two wave-wide rounds.
    int lo = 0, hi = a.n;                                  // answer in [lo, hi)
    while (hi - lo > 1) {
      const int span = hi - lo;
      const int step = (span + 63) / 64;
      const int idx = min(lo + lane * step, hi - 1);
      const bool le = a.item_start[idx] <= item && lo + lane * step < hi;
      const unsigned long long mask = __builtin_amdgcn_ballot_w64(le);
      const int cnt = __builtin_popcountll(mask);          // lanes 0 .. cnt-1 satisfy it (cnt >= 1)
      const int nlo = lo + (cnt - 1) * step;
      hi = min(nlo + step, hi);
      lo = nlo;
    }
    const int r = rfl(lo);
    const int rows = prefill_rows(a.n_q, a.lengths, a.q_start, a.total_q, r);
    const int len = a.lengths[r];
    const int n_blocks_item = (int)(((int64_t)rows * G + COLS_ITEM - 1) / COLS_ITEM);
    const int idx = item - a.item_start[r];
    const int g = idx / n_blocks_item;
    const int cb = n_blocks_item - 1 - (idx - g * n_blocks_item);    // heaviest (latest) columns first
    const int n_cols = rows * G;
    const int c0 = cb * COLS_ITEM + wv * COLS_WAVE;   // this wave's first column
    const bool active = c0 < n_cols;                                  // a wave without columns still helps to load
    const int64_t q_row0 = a.q_start[r];
    const int first_pos = len - rows;                                // position of query token 0

    // ---- per-lane columns: tile ct holds column c0 + 16 ct + col16
    int lim[CT];                                                       // keys visible to the column (0: column absent)
    const unsigned short* qptr[CT];
    bf16x8 qreg[CT][4];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const int col = c0 + 16 * ct + col16;
      const bool ok = col < n_cols;
      const int j = ok ? col / G : 0, h = ok ? col - j * G : 0;
      lim[ct] = ok ? first_pos + j + 1 : 0;
      qptr[ct] = a.q + ((q_row0 + j) * a.Hq + g * G + h) * 128;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        qreg[ct][s] = ok ? *(const bf16x8*)(qptr[ct] + 32 * s + 8 * g4) : z;
      }
    }
    // keys the item streams: up to the limit of its last column; this wave's own columns end earlier
    const int item_last_col = min((cb + 1) * COLS_ITEM, n_cols) - 1;
    const int item_lim_max = first_pos + item_last_col / G + 1;
    const int lim_min = first_pos + c0 / G + 1;                       // pairs below it need no mask in this wave
    const int n_tiles = (item_lim_max + BLK - 1) / BLK;
    const int n_pairs = (n_tiles + 1) / 2;

    float m[CT], lsum[CT];
    float4v O[CT][8];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      m[ct] = NEG_INF;
      lsum[ct] = 0.f;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) O[ct][dt] = float4v{0.f, 0.f, 0.f, 0.f};
    }

    const int64_t plane = (int64_t)g * a.head_stride;
    const const_i32* bt_row = as_constant(PAGED ? a.bt + (int64_t)r * a.bt_stride : nullptr);
    const int64_t base_block = PAGED ? 0 : a.offsets[r] / BLK;
    // ---- loading: this wave's tile of pair pr -> four 16-byte pieces per lane in registers -> LDS.  A
    // second tile that does not exist is written as zeros; V slots at or past `len` (stale bytes, maybe
    // NaN patterns) are zeroed too, so that a weight of 0 really removes them.  (K needs nothing: scores
    // of tokens past a column's limit are replaced, not multiplied.)
    auto tile_of = [&](int pr) { return 2 * pr + which; };
    int blk_next = 0;
    auto lookup = [&](int pr) {
      if (PAGED) blk_next = bt_row[min(tile_of(pr), n_tiles - 1)];
    };
    auto issue = [&](uint4v (&rg)[4], int pr) {
      const int t = min(tile_of(pr), n_tiles - 1);
      const int64_t off = plane + (PAGED ? (int64_t)blk_next : base_block + t) * TILE_BYTES;
#pragma unroll
      for (int s = 0; s < LOADS; ++s) rg[s] = *(const uint4v*)(src_base + off + s * 1024);
    };
    auto write_stage = [&](uint4v (&rg)[4], int pr) {
      char* st = stage_mem + (pr % PREFILL_STAGES) * PREFILL_STAGE_BYTES;
      const int t = tile_of(pr);
      const bool exists = t < n_tiles;
      if (FP8) {
        if (!loads_v) {
          // lane (t16, q) holds, per 64-channel half s, channels 64 s + 8 q .. +7 and 64 s + 32 + 8 q .. +7 of
          // token t16: two bf16 pieces, for channel octets 8 s + q and 8 s + 4 + q
#pragma unroll
          for (int s = 0; s < 2; ++s) {
            const uint4v w = exists ? rg[s] : uint4v{0u, 0u, 0u, 0u};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const uint4v o = {fp8x2_to_bf16x2<false>(w[2 * h]), fp8x2_to_bf16x2<true>(w[2 * h]),
                                fp8x2_to_bf16x2<false>(w[2 * h + 1]), fp8x2_to_bf16x2<true>(w[2 * h + 1])};
              *(uint4v*)(st + which * 4096 + (((8 * s + 4 * h + g4) * 16 + col16) * 16)) = o;
            }
          }
        } else {
          // lane (c, q) holds, per half s, one word per channel group 4 s + i: channel c of tokens 4q .. 4q+3
          const int tok0 = t * BLK + 4 * g4;
#pragma unroll
          for (int s = 0; s < 2; ++s) {
            const uint4v w = exists ? rg[s] : uint4v{0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              uint2v o = {fp8x2_to_bf16x2<false>(w[i]), fp8x2_to_bf16x2<true>(w[i])};
              if (tok0 + 4 > len) {                                     // some of the four tokens are not there
                if (tok0 + 0 >= len) o[0] &= 0xffff0000u;
                if (tok0 + 1 >= len) o[0] &= 0x0000ffffu;
                if (tok0 + 2 >= len) o[1] &= 0xffff0000u;
                if (tok0 + 3 >= len) o[1] &= 0x0000ffffu;
              }
              *(uint2v*)(st + 8192 + (4 * s + i) * 1024 + lane * 16 + which * 8) = o;
            }
          }
        }
      } else if (!loads_v) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
          *(uint4v*)(st + which * 4096 + s * 1024 + lane * 16) = exists ? rg[s] : uint4v{0u, 0u, 0u, 0u};
      } else {
        // lane (c, q) holds, per piece s, tokens 4q .. 4q+3 of channel groups 2s (low 8 bytes) and 2s+1
        const int tok0 = t * BLK + 4 * g4;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          uint4v w = exists ? rg[s] : uint4v{0u, 0u, 0u, 0u};
          if (tok0 + 4 > len) {                                       // some of the four tokens are not there
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (tok0 + i >= len) {
                const unsigned keep = (i & 1) ? 0x0000ffffu : 0xffff0000u;
                w[i >> 1] &= keep;
                w[2 + (i >> 1)] &= keep;
              }
          }
          char* dst = st + 8192 + lane * 16 + which * 8;
          *(uint2v*)(dst + (2 * s) * 1024) = uint2v{w[0], w[1]};
          *(uint2v*)(dst + (2 * s + 1) * 1024) = uint2v{w[2], w[3]};
        }
      }
    };

    // One pair of tiles against the wave's 64 columns.  Scores: S^T = K Q^T per tile (16x16x32 over
    // the channels).  O^T += V^T P^T contracts over the 32 tokens of the pair in one 16x16x32
    // instruction per channel group: lane (., g4) supplies tokens 4 g4 .. +3 of the first tile, then of
    // the second, which is how the score accumulators hold them and how the stage stores V.
    //
    // Softmax reference.  Softmax is invariant under the choice of the reference m subtracted in the
    // exponent, and fp32 / bf16 weights have room for 2^127: the fast pass fixes m of a column to the
    // exact maximum over the first pair (every column sees token 0) and never moves it, so the steady
    // state holds no cross-lane maximum, no rescale of O and no second exponential.  Should later scores
    // exceed that reference so far that a column's weight sum passes 2^90 (or turns inf / NaN), the item
    // is redone by the slow pass below, the classic online softmax that moves its references.
    auto scores = [&](float4v (&x)[CT][2], int pr) {
      const char* st = stage_mem + (pr % PREFILL_STAGES) * PREFILL_STAGE_BYTES + lane * 16;
      const int t0 = pr * 2 * BLK;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        bf16x8 kk[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) kk[s] = *(const bf16x8*)(st + b * 4096 + s * 1024);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          float4v s4 = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < 4; ++s) s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk[s], qreg[ct][s], s4, 0, 0, 0);
          x[ct][b] = s4;                                               // raw: the scale joins the exponent
        }
      }
      if (t0 + 2 * BLK > lim_min) {                                    // some column cannot see the whole pair
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (t0 + 16 * b + 4 * g4 + i >= lim[ct]) x[ct][b][i] = NEG_INF;
      }
    };
    // per-lane maximum of a column tile's eight scores, in exponent units (the scale is positive)
    auto lane_max = [&](const float4v (&xc)[2]) {
      return fmaxf(fmaxf(fmaxf(xc[0][0], xc[0][1]), fmaxf(xc[0][2], xc[0][3])),
                   fmaxf(fmaxf(xc[1][0], xc[1][1]), fmaxf(xc[1][2], xc[1][3]))) * a.scale_log2;
    };
    // the V operands of a pair: requested before the scores are computed, so that the LDS reads run under
    // the matrix instructions of S^T instead of in front of those of P V
    auto read_v = [&](bf16x8 (&av)[8], int pr) {
      const char* st = stage_mem + (pr % PREFILL_STAGES) * PREFILL_STAGE_BYTES + lane * 16;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) av[dt] = *(const bf16x8*)(st + 8192 + dt * 1024);
    };
    auto weights = [&](const float4v (&x)[CT][2], const bf16x8 (&av)[8]) {
      bf16x8 p8[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        float psum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(x[ct][b][i], a.scale_log2, -m[ct]));
            psum += pv;
            p8[ct][4 * b + i] = (__bf16)pv;
          }
        lsum[ct] += psum;
      }
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          O[ct][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dt], p8[ct], O[ct][dt], 0, 0, 0);
    };
    // fast pass: references fixed by the first pair.  m holds a finite value from then on (0 for a
    // column that does not exist).
    auto compute_fast = [&](int pr) {
      float4v x[CT][2];
      bf16x8 av[8];
      read_v(av, pr);
      scores(x, pr);
      if (pr == 0) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          float tmax = lane_max(x[ct]);
          tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
          tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
          m[ct] = tmax == NEG_INF ? 0.f : tmax;
        }
      }
      weights(x, av);
    };
    // slow pass: a reference moves whenever a score exceeds it by more than MAX_SLACK exponent units;
    // the sums and O are rescaled then.  m = -inf until a column has seen a score.
    constexpr float MAX_SLACK = 12.0f;
    auto compute_slow = [&](int pr) {
      float4v x[CT][2];
      scores(x, pr);
      bool moved = false;
      float local[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        local[ct] = lane_max(x[ct]);
        moved |= local[ct] > m[ct] + MAX_SLACK;                         // (m = -inf: any visible score moves it)
      }
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          float tmax = local[ct];
          tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
          tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
          const float m_new = fmaxf(m[ct], tmax);
          // a column that has seen nothing yet keeps m = -inf; 0 stands in so that no inf - inf appears
          const float alpha = __builtin_amdgcn_exp2f(m[ct] - (m_new == NEG_INF ? 0.f : m_new));
          lsum[ct] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) O[ct][dt] *= alpha;
          m[ct] = m_new;
        }
      }
      float keep[CT];
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        keep[ct] = m[ct];
        if (m[ct] == NEG_INF) m[ct] = 0.f;                              // stand-in while the weights are formed
      }
      bf16x8 av[8];
      read_v(av, pr);
      weights(x, av);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) m[ct] = keep[ct];
    };

    // ---- pipeline: the loads of pair p + 2 are in flight while pair p is computed; pair p + 1 sits in
    // registers until the computation of pair p is over, is written into the other stage, and one
    // work-group barrier per pair makes it visible (and tells that the stage of pair p is free again).
    auto stream = [&](auto&& compute) {
      uint4v ra[4], rb[4];
      lookup(0);
      issue(ra, 0);
      lookup(1);
      if (n_pairs > 1) issue(rb, 1);
      lookup(2);
      write_stage(ra, 0);
      __syncthreads();
      for (int pr = 0; pr < n_pairs; pr += 2) {
        if (pr + 2 < n_pairs) {
          issue(ra, pr + 2);
          lookup(pr + 3);
        }
        if (active) compute(pr);
        if (pr + 1 < n_pairs) write_stage(rb, pr + 1);
        __syncthreads();
        if (pr + 1 < n_pairs) {
          if (pr + 3 < n_pairs) {
            issue(rb, pr + 3);
            lookup(pr + 4);
          }
          if (active) compute(pr + 1);
          if (pr + 2 < n_pairs) write_stage(ra, pr + 2);
          __syncthreads();
        }
      }
    };
    // each lane summed the weights of its own tokens: a column's total is the sum over g4
    auto column_sums = [&](float (&l)[CT]) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        l[ct] = lsum[ct];
        l[ct] += __shfl_xor(l[ct], 16);
        l[ct] += __shfl_xor(l[ct], 32);
      }
    };

    float l[CT];
    stream(compute_fast);
    column_sums(l);
    bool redo = false;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) redo |= active && lim[ct] != 0 && !(l[ct] < 0x1p90f);
    if (threadIdx.x == 0) redo_slot = 0;
    __syncthreads();
    if (__builtin_amdgcn_ballot_w64(redo) != 0 && lane == 0) redo_slot = 1;
    __syncthreads();
    if (redo_slot != 0) {                                              // the whole work-group: the barriers are shared
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        m[ct] = NEG_INF;
        lsum[ct] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) O[ct][dt] = float4v{0.f, 0.f, 0.f, 0.f};
      }
      stream(compute_slow);
      column_sums(l);
    }
    if (!active) continue;

    // ---- normalise and store: lane (col16, g4) holds channels 16 dt + 4 g4 .. +3 of its columns
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      if (lim[ct] == 0) continue;
      const float inv = a.out_scale / l[ct];
      const int64_t o_base = (qptr[ct] - a.q) + 4 * g4;
      if (a.out_bf16) {
        unsigned short* o = (unsigned short*)a.out + o_base;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          uint2v pk;
          pk[0] = (unsigned)float_to_bf16_bits(O[ct][dt][0] * inv) | ((unsigned)float_to_bf16_bits(O[ct][dt][1] * inv) << 16);
          pk[1] = (unsigned)float_to_bf16_bits(O[ct][dt][2] * inv) | ((unsigned)float_to_bf16_bits(O[ct][dt][3] * inv) << 16);
          *(uint2v*)(o + 16 * dt) = pk;
        }
      } else {
        float* o = (float*)a.out + o_base;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *(float4v*)(o + 16 * dt) = O[ct][dt] * inv;
      }
    }
  }
}

}  // namespace
