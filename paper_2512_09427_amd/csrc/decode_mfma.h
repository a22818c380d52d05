// Matrix-core decode attention for bf16 storage (head_dim 128 or 64) and fp8 storage (head_dim 128), group size <= 16.
//
// Work decomposition ("tile stream").  A tile is one 16-token pool block of one KV head.
// All tiles of the batch form one sequence ordered by (request, KV head, block); the plan
// kernel cuts it into equal contiguous ranges, one per resident wavefront, so every wave
// streams the same number of bytes no matter how skewed the length distribution is.  A
// wave walks its range with two cursors: a prefetch cursor that issues the loads of the
// tile NBUF-1 steps ahead, and a compute cursor that consumes register buffers in order.
// The pipeline never drains at request boundaries.
//
// A (request, KV head) segment that lies inside one wave's range is finished by that wave
// and written straight to `out`.  A segment cut by a range boundary leaves un-normalised
// partial states (m, l, O).  The waves of a work-group (4 or 8) own consecutive ranges, so
// a cut between two of them is healed inside the work-group: the right-hand wave parks the
// state of its first piece in LDS as soon as that piece ends, and the left-hand wave, when
// it reaches the end of its range, folds that state into its own registers and writes the
// result.  Waves only ever wait for their right-hand neighbour, so the chain cannot
// deadlock and needs no barrier.  Only pieces cut by a work-group boundary go to the HBM
// workspace (at most two per work-group) and are merged by stream_reduce_kernel.
//
// Per tile:  S^T[16 tok x 16 heads] = K_blk[16 x 128] * Q^T[128 x 16]     4 x mfma 16x16x32 bf16
//            O^T[128 x 16 heads]   += V_blk^T[128 x 16 tok] * P^T[16 x 16] 8 x mfma 16x16x16 bf16
// Lane l holds column (query head) l%16 and rows 4*(l/16)..+3 of S^T, P^T and O^T, so the
// running max, the running sum and the rescale factor of a head live in the lanes that hold
// its column.  The pool's block format is exactly the MFMA operand order, so each wave-wide
// load is one contiguous KiB landing in the registers the MFMA reads.  P is split into
// bf16 hi + lo parts so the P*V product keeps about 16 bits of P.
#pragma once

#include <type_traits>

#include "kernels_common.h"

namespace {

using odma_plan::StreamEntry;
using odma_plan::WaveDesc;
using odma_plan::ReqPos;
using odma_plan::StreamHeader;
using odma_plan::ReduceDesc;
using odma_plan::STREAM_MAX_WG;

struct StreamArgs {
  const char* k;             // layer base of the K pool
  const char* v;
  const unsigned short* q;
  void* out;
  const void* k_new;         // fused step only: [n][Hkv][head_dim] rows (bf16, or E4M3 bytes) appended at position len-1
  const void* v_new;
  const int32_t* bt;
  int32_t bt_stride;
  const StreamHeader* hdr;
  const StreamEntry* entries;
  const WaveDesc* waves;
  const ReqPos* req_pos;
  const ReduceDesc* red;     // [n_workgroups + 1], the last one empty
  int32_t* arrive;           // [n_workgroups + 1] arrival counters of the in-kernel merge, zero between launches
  int32_t fuse_reduce;       // 1: the last work-group to finish a cut segment merges it; 0: stream_reduce_kernel does
  float2* part_ml;           // [2 * n_workgroups][Hq]
  float* part_o;             // [2 * n_workgroups][Hq][128]
  int32_t n, Hq, Hkv, G;
  int32_t wpw;               // waves per attention work-group (4 or 8)
  int32_t qs, aq;            // per-wave LDS queue depths: finished pieces, appended rows
  int64_t head_stride;       // bytes between KV-head planes of one layer
  float scale_log2;          // sm_scale * log2(e) (fp8 storage: times k_scale)
  int32_t head_dim;          // 128, or 64 (bf16 only): stride of q and out rows
  float out_scale;           // factor of the final normalisation: 1, or v_scale / 256 for fp8 storage (P is carried times 256)
  int32_t out_bf16;
};

constexpr int STREAM_PLAN_THREADS = 1024;
constexpr int STREAM_PLAN_LDS = 8192;

// ---------------------------------------------------------------------------------
// plan: lengths -> entries, per-request positions, one equal tile range per wave
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(STREAM_PLAN_THREADS) void stream_plan_kernel(
    const int32_t* __restrict__ lengths, const int64_t* __restrict__ offsets, int32_t n, int32_t Hkv,
    int32_t tile_tokens, int32_t n_waves, int32_t wpw, int32_t q_min, int32_t odd_xcd_weight, int32_t late_wave_weight,
    StreamHeader* hdr, StreamEntry* entries,
    WaveDesc* waves, ReqPos* req_pos, ReduceDesc* red, int32_t* arrive) {
  __shared__ int wave_tiles[STREAM_PLAN_THREADS / 64];
  __shared__ int wave_cnt[STREAM_PLAN_THREADS / 64];
  __shared__ int first_lds[STREAM_PLAN_LDS];
  __shared__ int wg_pos[STREAM_MAX_WG + 1];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (n + STREAM_PLAN_THREADS - 1) / STREAM_PLAN_THREADS;
  const int r0 = min(tid * per, n), r1 = min(r0 + per, n);
  int loc_tiles = 0, loc_cnt = 0;
  for (int r = r0; r < r1; ++r) {
    const int len = max(lengths[r], 0);
    loc_tiles += (len + tile_tokens - 1) / tile_tokens;
    loc_cnt += len > 0;
  }
  int inc_tiles = loc_tiles, inc_cnt = loc_cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int yt = __shfl_up(inc_tiles, o), yc = __shfl_up(inc_cnt, o);
    if (lane >= o) {
      inc_tiles += yt;
      inc_cnt += yc;
    }
  }
  if (lane == 63) {
    wave_tiles[wv] = inc_tiles;
    wave_cnt[wv] = inc_cnt;
  }
  __syncthreads();
  int base_tiles = 0, base_cnt = 0, sum_tiles = 0, n_entries = 0;
  for (int i = 0; i < STREAM_PLAN_THREADS / 64; ++i) {
    if (i < wv) {
      base_tiles += wave_tiles[i];
      base_cnt += wave_cnt[i];
    }
    sum_tiles += wave_tiles[i];
    n_entries += wave_cnt[i];
  }
  int run_tiles = base_tiles + inc_tiles - loc_tiles, run_cnt = base_cnt + inc_cnt - loc_cnt;
  const bool use_lds = n <= STREAM_PLAN_LDS;
  for (int r = r0; r < r1; ++r) {
    const int len = max(lengths[r], 0);
    const int tiles = (len + tile_tokens - 1) / tile_tokens;
    req_pos[r] = ReqPos{run_tiles * Hkv, tiles};
    if (len > 0) {
      StreamEntry e;
      e.r = r;
      e.tiles = tiles;
      e.first_pos = run_tiles * Hkv;
      e.len = len;
      e.base_block = offsets ? (int32_t)(offsets[r] / BLK) : 0;
      e.pad0 = e.pad1 = e.pad2 = 0;
      entries[run_cnt] = e;
      if (use_lds) first_lds[run_cnt] = e.first_pos;
      ++run_cnt;
    }
    run_tiles += tiles;
  }
  const int total = sum_tiles * Hkv;
  // one contiguous tile range per wave (rule and weights: odma_plan::StreamShares)
  const odma_plan::StreamShares shares = odma_plan::stream_shares(total, n_waves, wpw, q_min, odd_xcd_weight, late_wave_weight);
  const int used = shares.used;
  auto pos_of = [&](int W) -> int { return shares.start(W); };
  if (tid == 0) *hdr = StreamHeader{total, n_entries, n_waves, used};
  const int n_wg = n_waves / wpw;
  for (int b = tid; b <= n_wg; b += STREAM_PLAN_THREADS) wg_pos[b] = pos_of(b * wpw);   // work-group starts
  __threadfence_block();
  __syncthreads();
  auto entry_of = [&](int pos) -> int {                   // largest entry with first_pos <= pos
    int lo = 0, hi = n_entries - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      const int f = use_lds ? first_lds[mid] : entries[mid].first_pos;
      if (f <= pos) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  for (int w = tid; w < n_waves; w += STREAM_PLAN_THREADS) {
    const int ps = pos_of(w), pe = pos_of(w + 1);
    WaveDesc wd;
    wd.pos_start = ps;
    wd.pos_end = pe;
    wd.entry0 = 0;
    wd.n_entries = n_entries;
    wd.r = wd.tiles = wd.first_pos = wd.len = wd.base_block = wd.r_next = wd.pad1 = wd.pad2 = 0;
    if (ps < pe) {
      const int lo = entry_of(ps);
      const StreamEntry e = entries[lo];
      wd.entry0 = lo;
      wd.r = e.r;
      wd.tiles = e.tiles;
      wd.first_pos = e.first_pos;
      wd.len = e.len;
      wd.base_block = e.base_block;
      wd.r_next = entries[min(lo + 1, n_entries - 1)].r;
    }
    waves[w] = wd;
  }
  // merge work: the boundary in front of work-group b cuts a segment iff the segment starts
  // before it; the first boundary inside a segment owns the merge of all its partials
  auto wg_of = [&](int pos) -> int {                      // work-group whose range holds pos (pos < total)
    int lo = 0, hi = used / wpw - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (wg_pos[mid] <= pos) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  for (int b = tid; b <= n_wg; b += STREAM_PLAN_THREADS) {
    ReduceDesc rd = {0, 0, 0, 0};
    const int bpos = wg_pos[min(b, n_wg)];
    if (b > 0 && b < n_wg && bpos < total) {
      const StreamEntry e = entries[entry_of(bpos)];
      const int g = (bpos - e.first_pos) / e.tiles;
      const int start = e.first_pos + g * e.tiles;
      if (start < bpos) {
        rd.b0 = wg_of(start);
        rd.n_parts = wg_of(start + e.tiles - 1) - rd.b0 + 1;
        rd.r = e.r;
        rd.g = g;
      }
    }
    red[b] = rd;
    arrive[b] = 0;
  }
}

// ---------------------------------------------------------------------------------
// attention over one tile stream per wave
// ---------------------------------------------------------------------------------

// LDS per work-group: one hand-off slot per wave (O[G][128], m[G], l[G], padded; slot 0 unused),
// {ready, to_end} per wave, then per wave a queue of finished pieces waiting to be written to
// global memory (qs entries of slot + 8 ints) and of appended rows (aq records of STREAM_AQ_INTS).  The host sizes
// the queues to the tiles a wave gets: a wave that runs out of queue has to write in mid-stream.
constexpr int STREAM_MERGE_BATCH = 16;   // most partials whose loads are in flight together in the in-kernel merge
__host__ __device__ inline int stream_slot_floats(int G) { return G * 128 + ((2 * G + 3) & ~3); }
constexpr int STREAM_AQ_INTS = 8 + 128 + 256;   // appended-row record: 8 ints of header, 512 B of K pieces, 1 KiB of V pieces
__host__ __device__ inline int stream_wave_queue_floats(int G, int qs, int aq) {
  return qs * (stream_slot_floats(G) + 8) + aq * STREAM_AQ_INTS;
}
__host__ inline size_t stream_lds_bytes(int G, int wpw, int qs, int aq) {
  return ((size_t)wpw * stream_slot_floats(G) + 2 * wpw + (size_t)wpw * stream_wave_queue_floats(G, qs, aq)) * 4;
}


// Partial states cross from one XCD's L2 to another's inside one launch.  They are written and
// read with agent-scope accesses (write-through / coherent reads, 8 bytes at a time), which keeps
// the exchange coherent without flushing or invalidating a whole L2 -- a release or acquire fence
// at agent scope does exactly that on this part and costs tens of microseconds per launch.
__device__ __forceinline__ void store_pair_agent(float* p, float x, float y) {
  const unsigned long long v = (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32);
  __hip_atomic_store((unsigned long long*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_pair_agent(const float* p) {
  const unsigned long long v = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}

// Maximum over the four lanes that hold one column (lanes l, l ^ 16, l ^ 32, l ^ 48), in every one of them: two
// register swaps between rows of 16 lanes and between halves of the wave, no trip through the LDS crossbar.
__device__ __forceinline__ float column_max(float x) {
  const unsigned u = __float_as_uint(x);
  const uint2v r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  const unsigned w = __float_as_uint(y);
  const uint2v h = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
}
__device__ __forceinline__ float column_sum(float x) {
  const unsigned u = __float_as_uint(x);
  const uint2v r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  const unsigned w = __float_as_uint(y);
  const uint2v h = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(h[0]) + __uint_as_float(h[1]);
}
constexpr float LAZY_REF_LOG2 = 8.0f;

// Development builds only (-DODMA_DEV_TIMELINE): wall-clock stamps (100 MHz) per wave, read back with
// odma_dev_timeline().  Slots: 0 kernel entry, 1 range descriptor in registers, 2 stream end, 3 queued results written,
// 4 work-group end, 5 tiles streamed, 8 + i: tile i consumed.
#ifdef ODMA_DEV_TIMELINE
constexpr int TL_SLOTS = 64;
__device__ long long odma_dev_timeline_buf[4096 * TL_SLOTS];
#define TL_STAMP(slot) do { if (lane == 0 && (slot) < TL_SLOTS) tl_lds[wv][(slot)] = wall_clock64(); } while (0)
#else
#define TL_STAMP(slot) do { } while (0)
#endif

struct Window {              // 64 consecutive entries, one per lane
  int r, tiles, len, base_block;
  int r_next;                // request of the entry after this lane's
};

struct Cursor {              // wave-uniform position in the tile stream
  int e_base, ei;            // entry = e_base + ei, ei indexes the lane window
  int g, t;                  // KV head and block inside the request
  int r, tiles, len, base_block;
  int r_next;                // request of the following entry
  int blk;                   // paged layout: physical block of the cursor's tile, fetched one step ahead
  int blk2;                  // fp8, paged: the tile's second block
};

// storage formats served by the tile stream
constexpr int STREAM_BF16_D128 = 0, STREAM_FP8_D128 = 1, STREAM_BF16_D64 = 2;

template <bool PAGED, int NBUF, int WPW, bool FUSED, int FMT>
__global__ __launch_bounds__(64 * WPW, 2) void decode_stream_kernel(StreamArgs a) {
  constexpr bool FP8 = FMT == STREAM_FP8_D128, D64 = FMT == STREAM_BF16_D64;
  constexpr bool TWO = FMT != STREAM_BF16_D128;              // blocks of 2 KiB: a tile is two of them
  constexpr int HD = D64 ? 64 : 128;                         // head_dim: stride of q and out rows
  // A tile is what a wave requests per step: 4 KiB of K and 4 KiB of V.  bf16 with head_dim 128: one
  // 16-token pool block; fp8, or bf16 with head_dim 64: two of them (32 tokens), which need not be
  // neighbours in the paged layout.  (Inside the kernel every state keeps 128 channels per head; with
  // head_dim 64 the upper half stays zero and is not written out.)
  constexpr int TT = TWO ? 32 : BLK;
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int col = lane & 15, g4 = lane >> 4;
  const int G = a.G, Hkv = a.Hkv;
  const int slot_floats = stream_slot_floats(G);
  // [wave]{ready, to_end}; read and written with work-group-scope atomics (plain LDS instructions:
  // a volatile access would be compiled as a FLAT one, which also waits for the tile loads in flight)
  int* flags = (int*)(lds + WPW * slot_floats);
  auto flag_set = [&](int i, int v) { __hip_atomic_store(flags + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); };
  auto flag_get = [&](int i) -> int { return __hip_atomic_load(flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); };
  const float NEG_INF = -INFINITY;
#ifdef ODMA_DEV_TIMELINE
  __shared__ long long tl_lds[WPW][TL_SLOTS];
  if (lane < TL_SLOTS) tl_lds[wv][lane] = 0;
  TL_STAMP(0);
#endif
  constexpr int BLOCK_BYTES = BLK * HD * (FP8 ? 1 : 2);    // one pool block of K (or V)

  // the wave's range first: everything else waits for it
  const WaveDesc wd = a.waves[blockIdx.x * WPW + rfl(wv)];
  // in-kernel merge: the segments cut at this work-group's two boundaries, requested now so that the
  // epilogue does not wait for them
  ReduceDesc rd_cut[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
  if (a.fuse_reduce) {
    rd_cut[0] = a.red[blockIdx.x];
    rd_cut[1] = a.red[blockIdx.x + 1];
  }
  // requested early, needed last: whether the request this thread looks after is empty
  const int r_mine = blockIdx.x * (64 * WPW) + threadIdx.x;
  const int tiles_mine = r_mine < a.n ? a.req_pos[r_mine].tiles : 1;
  const int pos_start = rfl(wd.pos_start), pos_end = rfl(wd.pos_end), n_entries = rfl(wd.n_entries);
  const int n_my = pos_end - pos_start;
  TL_STAMP(1);
  // ready flags must be clear before any neighbour can look at them: a wave clears its own
  // flag first thing, and its left neighbour reads it only at the end of a whole tile range,
  // so one work-group barrier at the top settles the order
  if (lane == 0) flag_set(2 * wv, 0);
  __syncthreads();

  if (n_my > 0) {
    const char* kbase = a.k + lane * 16;
    const char* vbase = a.v + lane * 16;

    auto load_window = [&](Window& w, int e_base) {
      const int idx = min(e_base + lane, n_entries - 1);
      const int4 lo = *(const int4*)&a.entries[idx];
      w.r = lo.x;
      w.tiles = lo.y;
      w.len = lo.w;
      w.base_block = a.entries[idx].base_block;
      w.r_next = a.entries[min(idx + 1, n_entries - 1)].r;
    };
    auto fetch = [&](Cursor& c, const Window& w) {
      c.r = __builtin_amdgcn_readlane(w.r, c.ei);
      c.tiles = __builtin_amdgcn_readlane(w.tiles, c.ei);
      c.len = __builtin_amdgcn_readlane(w.len, c.ei);
      c.base_block = __builtin_amdgcn_readlane(w.base_block, c.ei);
      c.r_next = __builtin_amdgcn_readlane(w.r_next, c.ei);   // every window register is read here, so
    };                                                          // none stays pending after a reload
    auto advance = [&](Cursor& c, Window& w) {
      if (++c.t == c.tiles) {
        c.t = 0;
        if (++c.g == Hkv) {
          c.g = 0;
          if (++c.ei == 64) {
            c.e_base += 64;
            c.ei = 0;
            load_window(w, c.e_base);
          }
          fetch(c, w);
        }
      }
    };
    // Paged layout: the block id of a tile is one dependent (scalar) load away from its address.
    // The prefetch cursor asks for it right after it moves, a whole step before the tile's loads
    // are issued, so the table look-up never sits in front of them.
    auto lookup_block = [&](Cursor& c) {
      if (PAGED) {
        const const_i32* row = as_constant(a.bt + (int64_t)c.r * a.bt_stride);
        if (TWO) {
          const int second = 2 * c.t + 1 < (c.len + BLK - 1) / BLK ? 2 * c.t + 1 : 2 * c.t;   // a last tile may have one block
          c.blk = row[2 * c.t];
          c.blk2 = row[second];
        } else {
          c.blk = row[c.t];
        }
      }
    };
    // physical byte offset of the cursor's tile inside a KV-head plane (fp8: of its first block)
    auto tile_offset = [&](const Cursor& c) -> int64_t {
      const int64_t blk = PAGED ? (int64_t)c.blk : (int64_t)c.base_block + c.t * (TT / BLK);
      return (int64_t)c.g * a.head_stride + blk * BLOCK_BYTES;
    };
    // fp8: byte offset of the tile's second block.  A last tile that holds 16 tokens or fewer has
    // none: its loads re-read the first block, so nothing outside the request's slab is touched.
    auto tile_offset2 = [&](const Cursor& c) -> int64_t {
      if (PAGED) return (int64_t)c.g * a.head_stride + (int64_t)c.blk2 * BLOCK_BYTES;
      const bool has = 2 * c.t + 1 < (c.len + BLK - 1) / BLK;
      return (int64_t)c.g * a.head_stride + ((int64_t)c.base_block + 2 * c.t + (has ? 1 : 0)) * BLOCK_BYTES;
    };

    Window wc, wp;                                         // compute and prefetch windows
    Cursor cc, pc;
    cc.e_base = rfl(wd.entry0);
    cc.ei = 0;
    cc.r = rfl(wd.r);
    cc.tiles = rfl(wd.tiles);
    cc.len = rfl(wd.len);
    cc.base_block = rfl(wd.base_block);
    cc.r_next = rfl(wd.r_next);
    {
      const int rel = pos_start - rfl(wd.first_pos);
      cc.g = rel / cc.tiles;
      cc.t = rel - cc.g * cc.tiles;
    }
    cc.blk = 0;
    pc = cc;
    lookup_block(pc);
    load_window(wc, cc.e_base);                            // needed only when a cursor leaves the first entry
    wp = wc;

    bf16x8 kb[NBUF][4], vb[NBUF][4];
    // Loads of the prefetch cursor's tile.  They are issued in every step, so that the waits stay
    // static counts; once the whole range has been requested the surplus loads all read the first
    // block of the layer's pools, which stays in the L2 instead of costing HBM traffic.
    int to_issue = n_my;
    auto issue = [&](bf16x8 (&kk)[4], bf16x8 (&vv)[4]) {
      const int64_t off = to_issue > 0 ? tile_offset(pc) : 0;
      // fp8: loads 0, 1 read the first block of the tile, loads 2, 3 the second one
      const int64_t off2 = !TWO ? off + 2048 : (to_issue > 0 ? tile_offset2(pc) : 0);
      --to_issue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // streaming loads: K/V bytes are used once, and loads that do not allocate in the caches
        // read 9 % faster on this part (measured)
        const int64_t o = j < 2 ? off + j * 1024 : off2 + (j - 2) * 1024;
        kk[j] = __builtin_nontemporal_load((const bf16x8*)(kbase + o));
        vv[j] = __builtin_nontemporal_load((const bf16x8*)(vbase + o));
      }
    };
    // Q^T operand of the segment at cursor c: lane (col, g4) holds q[head col][32 j + 8 g4 .. +8]
    auto load_q = [&](bf16x8 (&qq)[4], int r, int g) {
      const bf16x8* qp = (const bf16x8*)(a.q + ((int64_t)r * a.Hq + g * G + col) * HD + 8 * g4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        qq[j] = (col < G && 32 * j < HD) ? qp[4 * j] : z;
      }
    };

    // The first segment's queries are requested ahead of the first tiles and adopted inside the main loop, after
    // the second tile's loads have been issued: waiting for them here would hold those loads back by a whole
    // memory round trip.
    bf16x8 qreg[4], qnext[4];
    load_q(qnext, cc.r, cc.g);

    // prologue: NBUF-1 tiles in flight
    int p_left = n_my - 1;                                 // prefetch cursor may still advance this often
#pragma unroll
    for (int d = 0; d < NBUF - 1; ++d) {
      issue(kb[d], vb[d]);
      if (p_left > 0) {
        advance(pc, wp);
        lookup_block(pc);
        --p_left;
      }
    }
    // fp8 storage: the queries go to the matrix cores as fp8 too.  Each query row is scaled by a
    // power of two that brings its largest magnitude into [128, 256) and split into a high and a
    // low E4M3 part (together about 8 significant bits); the inverse scale joins the softmax scale.
    long qhi[4] = {0, 0, 0, 0}, qlo[4] = {0, 0, 0, 0};
    float qfac = a.scale_log2;
    auto adopt_q = [&](const bf16x8 (&src)[4]) {
      if (!FP8) {
#pragma unroll
        for (int j = 0; j < 4; ++j) qreg[j] = src[j];
        return;
      }
      float qf[4][8];
      float amax = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          qf[j][i] = (float)src[j][i];
          amax = fmaxf(amax, fabsf(qf[j][i]));
        }
      amax = column_max(amax);
      const int ex = (int)((__float_as_uint(amax) >> 23) & 0xffu);     // amax in [2^(ex-127), 2^(ex-126))
      const bool tiny = ex < 16;                                        // zero or next to it: leave unscaled
      const float qs = tiny ? 1.0f : __uint_as_float((unsigned)(261 - ex) << 23);     // 2^(134 - ex)
      const float qs_inv = tiny ? 1.0f : __uint_as_float((unsigned)(ex - 7) << 23);
      qfac = a.scale_log2 * qs_inv;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int hi[2], lo[2];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          const float x0 = qf[j][4 * w] * qs, x1 = qf[j][4 * w + 1] * qs, x2 = qf[j][4 * w + 2] * qs, x3 = qf[j][4 * w + 3] * qs;
          int h = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
          h = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, h, true);
          int l = __builtin_amdgcn_cvt_pk_fp8_f32(x0 - __builtin_amdgcn_cvt_f32_fp8(h, 0), x1 - __builtin_amdgcn_cvt_f32_fp8(h, 1), 0, false);
          l = __builtin_amdgcn_cvt_pk_fp8_f32(x2 - __builtin_amdgcn_cvt_f32_fp8(h, 2), x3 - __builtin_amdgcn_cvt_f32_fp8(h, 3), l, true);
          hi[w] = h;
          lo[w] = l;
        }
        qhi[j] = (long)(unsigned)hi[0] | ((long)hi[1] << 32);
        qlo[j] = (long)(unsigned)lo[0] | ((long)lo[1] << 32);
      }
    };
    float m = NEG_INF, lsum = 0.f;
    float4v O[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) O[i] = float4v{0.f, 0.f, 0.f, 0.f};
    bool from_start = cc.t == 0;

    // fused step: the token appended this step is the last token of its segment.  Its K/V row
    // comes from k_new/v_new, is patched into the registers of the segment's last tile and is
    // written into the pool by the wave that owns that tile (no other wave touches the slot).
    // The row is fetched with one wave-wide load (lanes 0..31 the K row, lanes 32..63 the V row,
    // 8 bytes each; 128-byte rows -- fp8 storage, or bf16 with head_dim 64: 4 bytes each) and handed to
    // the lanes that need its pieces through LDS: one entry in the load queue per segment instead of twelve.
    uint2v newrow = {0u, 0u};
    bool new_ready = false;
    auto load_new = [&](int r, int g) {
      const char* base = (const char*)(lane < 32 ? a.k_new : a.v_new);
      if (TWO) newrow[0] = *(const unsigned*)(base + ((int64_t)r * Hkv + g) * 128 + 4 * (lane & 31));
      else newrow = *(const uint2v*)(base + ((int64_t)r * Hkv + g) * 256 + 8 * (lane & 31));
    };
    // The patch happens in registers now; the write into the pool is queued in LDS and done after
    // the range has been streamed, for the same reason as the outputs.  What is written back is not
    // the bare row (16-byte pieces of K, 2-byte pieces of V: partial sectors, which the memory side
    // turns into read-modify-writes) but the patched registers that hold it: the K pieces of the
    // token pair {slot, slot^1} (32-byte sectors) and the V pieces of the token quad slot/4 (whole
    // 256-byte runs).  The neighbours' bytes go back unchanged; slots past the end may get stale
    // bytes again, as before.  fp8 storage: the same with the 2 KiB block that holds the token (two
    // 1 KiB pieces of K and of V instead of four).
    constexpr int NP = TWO ? 2 : 4;                          // 1 KiB pieces per pool block
    int* abase = (int*)(lds + WPW * slot_floats + 2 * WPW + wv * stream_wave_queue_floats(G, a.qs, a.aq) +
                        a.qs * (slot_floats + 8));
    int an = 0;
    // (Results leave with streaming stores: ordinary ones stay in the L2 as dirty lines that the end
    // of the kernel has to write back, which showed as 0.8 us per launch.)
    auto flush_appends = [&]() {
      for (int i = 0; i < an; ++i) {
        const int* rec = abase + i * STREAM_AQ_INTS;
        const int64_t off = ((int64_t)rfl(rec[1]) << 32) | (unsigned)rfl(rec[0]);
        const int slot = rfl(rec[2]);
        const bf16x8* kq = (const bf16x8*)(rec + 8);
        const bf16x8* vq = (const bf16x8*)(rec + 8 + 128);
        if ((col >> 1) == (slot >> 1)) {
          char* kd = (char*)a.k + off + lane * 16;
#pragma unroll
          for (int j = 0; j < NP; ++j) __builtin_nontemporal_store(kq[(j * 4 + g4) * 2 + (col & 1)], (bf16x8*)(kd + j * 1024));
        }
        if (g4 == (slot >> 2)) {
          char* vd = (char*)a.v + off + lane * 16;
#pragma unroll
          for (int j = 0; j < NP; ++j) __builtin_nontemporal_store(vq[j * 16 + col], (bf16x8*)(vd + j * 1024));
        }
      }
      an = 0;
    };
    // Blocks of 2 KiB (fp8 storage, or bf16 with head_dim 64): the row's 128 K bytes and 128 V bytes are
    // staged in the unused upper half of the record's K area; k0, k1 / v0, v1 are the register pieces of
    // the block that holds the token.
    auto patch_two = [&](int* rec, int slot, bf16x8& k0, bf16x8& k1, bf16x8& v0, bf16x8& v1) {
      typedef unsigned uint4u __attribute__((ext_vector_type(4)));
      const int rr = slot & 3;
      unsigned* stage = (unsigned*)(rec + 8 + 64);
      stage[lane] = newrow[0];
      if (FP8) {
        const uint2v* krow = (const uint2v*)stage;          // K[0..128) as 16 pieces of 8 bytes
        const unsigned char* vrow = (const unsigned char*)(stage + 32);
        if (col == slot) {                                   // K: per 64-channel half, 8 channels of each of its two k-steps
          const uint2v a0 = krow[g4], b0 = krow[4 + g4], a1 = krow[8 + g4], b1 = krow[12 + g4];
          k0 = __builtin_bit_cast(bf16x8, uint4u{a0[0], a0[1], b0[0], b0[1]});
          k1 = __builtin_bit_cast(bf16x8, uint4u{a1[0], a1[1], b1[0], b1[1]});
        }
        if (g4 == (slot >> 2)) {                             // V: byte rr of every word is the new token's channel
          uint4u w0 = __builtin_bit_cast(uint4u, v0), w1 = __builtin_bit_cast(uint4u, v1);
          const unsigned keep = ~(0xffu << (8 * rr));
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            w0[w] = (w0[w] & keep) | ((unsigned)vrow[16 * w + col] << (8 * rr));
            w1[w] = (w1[w] & keep) | ((unsigned)vrow[64 + 16 * w + col] << (8 * rr));
          }
          v0 = __builtin_bit_cast(bf16x8, w0);
          v1 = __builtin_bit_cast(bf16x8, w1);
        }
      } else {
        const bf16x8* krow = (const bf16x8*)stage;          // K[0..64) as 8 pieces of 8 channels
        const unsigned short* vrow = (const unsigned short*)(stage + 32);
        if (col == slot) {                                   // K: 8 channels of the new token per k-step
          k0 = krow[g4];
          k1 = krow[4 + g4];
        }
        if (g4 == (slot >> 2)) {                             // V: this lane holds tokens 4*g4..+3 of 4 channels
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const __bf16 vnew = __builtin_bit_cast(__bf16, vrow[16 * k + col]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (i == rr) {
                if (k < 2) v0[4 * (k & 1) + i] = vnew;
                else v1[4 * (k & 1) + i] = vnew;
              }
          }
        }
      }
      if ((col >> 1) == (slot >> 1)) {                       // K pieces of the token pair, patched
        bf16x8* kq = (bf16x8*)(rec + 8);
        kq[g4 * 2 + (col & 1)] = k0;
        kq[(4 + g4) * 2 + (col & 1)] = k1;
      }
      if (g4 == (slot >> 2)) {                               // V pieces of the token quad, patched
        bf16x8* vq = (bf16x8*)(rec + 8 + 128);
        vq[col] = v0;
        vq[16 + col] = v1;
      }
    };
    auto patch_and_store = [&](bf16x8 (&kk)[4], bf16x8 (&vv)[4]) {
      const int slot = (cc.len - 1) & (BLK - 1), rr = slot & 3;
      lookup_block(cc);                                      // the compute cursor looks its block up only here
      const bool second = TWO && (((cc.len - 1) / BLK) & 1);  // 32-token tiles: the token sits in the tile's second block
      const int64_t off = second ? tile_offset2(cc) : tile_offset(cc);
      if (an == a.aq) flush_appends();
      int* rec = abase + an * STREAM_AQ_INTS;
      if (lane == 0) {
        rec[0] = (int)(off & 0xffffffffll);
        rec[1] = (int)(off >> 32);
        rec[2] = slot;
      }
      ++an;
      if (TWO) {
        if (second) patch_two(rec, slot, kk[2], kk[3], vv[2], vv[3]);
        else patch_two(rec, slot, kk[0], kk[1], vv[0], vv[1]);
        return;
      }
      // stage the row in the record's V area (overwritten by the patched pieces further down)
      uint2v* stage = (uint2v*)(rec + 8 + 128);
      stage[lane] = newrow;
      const bf16x8* krow = (const bf16x8*)stage;            // K[0..128) as 16 pieces of 8
      const unsigned short* vrow = (const unsigned short*)stage + 128;
      if (col == slot) {                                     // K: this lane holds 8 channels of the new token per k-step
#pragma unroll
        for (int j = 0; j < 4; ++j) kk[j] = krow[4 * j + g4];
      }
      if (g4 == (slot >> 2)) {                               // V: this lane holds tokens 4*g4..+3 of 8 channels
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const __bf16 vnew = __builtin_bit_cast(__bf16, vrow[16 * k + col]);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (i == rr) vv[k >> 1][4 * (k & 1) + i] = vnew;
        }
      }
      if ((col >> 1) == (slot >> 1)) {                       // K pieces of the token pair, patched
        bf16x8* kq = (bf16x8*)(rec + 8);
#pragma unroll
        for (int j = 0; j < 4; ++j) kq[(j * 4 + g4) * 2 + (col & 1)] = kk[j];
      }
      if (g4 == (slot >> 2)) {                               // V pieces of the token quad, patched
        bf16x8* vq = (bf16x8*)(rec + 8 + 128);
#pragma unroll
        for (int j = 0; j < 4; ++j) vq[j * 16 + col] = vv[j];
      }
    };

    // fp8 tile: 32 tokens in two pool blocks b = 0, 1.  Per block S^T = K Q^T with the high and the
    // low part of Q (2 x 4 mfma 16x16x32 fp8).  P is carried times 256 and split into a high and a
    // low E4M3 part as well; O^T += V^T P^T contracts over all 32 tokens in one mfma per d-tile and
    // part, the operand of lane (., g4) holding tokens 4 g4 .. 4 g4 + 3 of block 0, then of block 1,
    // which is the order the pool's V block format and the S^T accumulator layout both give.
    auto compute_fp8 = [&](bf16x8 (&kk)[4], bf16x8 (&vv)[4]) {
      typedef long long2v __attribute__((ext_vector_type(2)));
      typedef unsigned uint4u __attribute__((ext_vector_type(4)));
      const int n_valid = cc.len - cc.t * TT;               // tokens of this tile in range (>= 32: all)
      const bool ragged = n_valid < TT;
      float x[2][4];
      float tmax = NEG_INF;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float4v s = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const long kop = __builtin_bit_cast(long2v, kk[2 * b + (j >> 1)])[j & 1];
          s = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(kop, qhi[j], s, 0, 0, 0);
          s = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(kop, qlo[j], s, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float val = s[i] * qfac;
          if (ragged && 16 * b + 4 * g4 + i >= n_valid) val = NEG_INF;
          x[b][i] = val;
          tmax = fmaxf(tmax, val);
        }
      }
      tmax = column_max(tmax);
      // weights are carried times 256 in E4M3 (largest value 448), so the reference must be the exact running maximum;
      // the rescale is skipped when no column's maximum moved
      if (__builtin_amdgcn_ballot_w64(tmax > m) != 0) {
        const float m_new = fmaxf(m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) O[i] *= alpha;
      }
      float psum = 0.f;
      int ph[2], pl[2];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float pv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          pv[i] = __builtin_amdgcn_exp2f(x[b][i] - m);
          psum += pv[i];
          pv[i] *= 256.0f;
        }
        int h = __builtin_amdgcn_cvt_pk_fp8_f32(pv[0], pv[1], 0, false);
        h = __builtin_amdgcn_cvt_pk_fp8_f32(pv[2], pv[3], h, true);
        int l = __builtin_amdgcn_cvt_pk_fp8_f32(pv[0] - __builtin_amdgcn_cvt_f32_fp8(h, 0), pv[1] - __builtin_amdgcn_cvt_f32_fp8(h, 1), 0, false);
        l = __builtin_amdgcn_cvt_pk_fp8_f32(pv[2] - __builtin_amdgcn_cvt_f32_fp8(h, 2), pv[3] - __builtin_amdgcn_cvt_f32_fp8(h, 3), l, true);
        ph[b] = h;
        pl[b] = l;
      }
      lsum += psum;
      const long phi = (long)(unsigned)ph[0] | ((long)ph[1] << 32);
      const long plo = (long)(unsigned)pl[0] | ((long)pl[1] << 32);
      // bytes of tokens past the end may hold anything (0x7f is a NaN): keep 0 * x == 0
      unsigned keep0 = 0xffffffffu, keep1 = 0xffffffffu;
      if (ragged) {
        const int v0 = min(max(n_valid - 4 * g4, 0), 4), v1 = min(max(n_valid - 16 - 4 * g4, 0), 4);
        keep0 = v0 == 4 ? 0xffffffffu : (1u << (8 * v0)) - 1u;
        keep1 = v1 == 4 ? 0xffffffffu : (1u << (8 * v1)) - 1u;
      }
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const unsigned w0 = __builtin_bit_cast(uint4u, vv[dt >> 2])[dt & 3] & keep0;
        const unsigned w1 = __builtin_bit_cast(uint4u, vv[2 + (dt >> 2)])[dt & 3] & keep1;
        const long av = (long)w0 | ((long)w1 << 32);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(av, phi, O[dt], 0, 0, 0);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(av, plo, O[dt], 0, 0, 0);
      }
    };

    // bf16, head_dim 64: the tile is two pool blocks of 2 KiB (32 tokens), kk / vv [0], [1] the two
    // 1 KiB pieces of the first block, [2], [3] those of the second.  Scores per block as for head_dim
    // 128 with two channel steps; P V contracts over the 32 tokens in one 16x16x32 instruction per
    // channel group, the operand of lane (., g4) holding tokens 4 g4 .. +3 of the first block, then of
    // the second.  P is carried as a high plus a low bf16 part.
    auto compute_d64 = [&](bf16x8 (&kk)[4], bf16x8 (&vv)[4]) {
      const int n_valid = cc.len - cc.t * TT;               // tokens of this tile in range (>= 32: all)
      const bool ragged = n_valid < TT;
      float x[2][4];
      float tmax = NEG_INF;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float4v s = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 2; ++j) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk[2 * b + j], qreg[j], s, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float val = s[i] * a.scale_log2;
          if (ragged && 16 * b + 4 * g4 + i >= n_valid) val = NEG_INF;
          x[b][i] = val;
          tmax = fmaxf(tmax, val);
        }
      }
      tmax = column_max(tmax);
      if (__builtin_amdgcn_ballot_w64(tmax > m + LAZY_REF_LOG2) != 0) {   // lazy reference, as for head_dim 128
        const float m_new = fmaxf(m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i) O[i] *= alpha;
      }
      float psum = 0.f;
      bf16x8 phi, plo;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float pv = __builtin_amdgcn_exp2f(x[b][i] - m);
          psum += pv;
          const __bf16 hi = (__bf16)pv;
          phi[4 * b + i] = hi;
          plo[4 * b + i] = (__bf16)(pv - (float)hi);
        }
      lsum += psum;
      if (ragged) {
        // slots past the end may hold stale bytes (even NaN patterns): zero them so 0 * x stays 0
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (16 * b + 4 * g4 + i >= n_valid) {
                vv[2 * b + j][i] = (__bf16)0.f;
                vv[2 * b + j][4 + i] = (__bf16)0.f;
              }
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 wa = vv[dt >> 1], wb = vv[2 + (dt >> 1)];
        const bf16x8 av = (dt & 1) ? bf16x8{wa[4], wa[5], wa[6], wa[7], wb[4], wb[5], wb[6], wb[7]}
                                   : bf16x8{wa[0], wa[1], wa[2], wa[3], wb[0], wb[1], wb[2], wb[3]};
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, phi, O[dt], 0, 0, 0);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, plo, O[dt], 0, 0, 0);
      }
    };

    auto compute = [&](bf16x8 (&kk)[4], bf16x8 (&vv)[4]) {
      if (FP8) {
        compute_fp8(kk, vv);
        return;
      }
      if (D64) {
        compute_d64(kk, vv);
        return;
      }
      float4v s = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk[j], qreg[j], s, 0, 0, 0);
      const int n_valid = cc.len - cc.t * BLK;              // tokens of this block in range (>= 16: all)
      const bool ragged = n_valid < BLK;
      float x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = s[i] * a.scale_log2;
      if (ragged) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (4 * g4 + i >= n_valid) x[i] = NEG_INF;
      }
      const float tmax = column_max(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])));
      // The reference of the running softmax moves only when a column's scores pass it by more than 2^LAZY_REF_LOG2:
      // the state (m, l, O) is valid for any reference, weights up to 2^LAZY_REF_LOG2 are exact enough in fp32 and in the
      // high + low bf16 pair, and the usual tile then needs no rescale of O and no second exponential.
      if (__builtin_amdgcn_ballot_w64(tmax > m + LAZY_REF_LOG2) != 0) {
        const float m_new = fmaxf(m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) O[i] *= alpha;
      }
      float psum = 0.f;
      bf16x4 phi, plo;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float pv = __builtin_amdgcn_exp2f(x[i] - m);
        psum += pv;
        const __bf16 hi = (__bf16)pv;
        phi[i] = hi;
        plo[i] = (__bf16)(pv - (float)hi);
      }
      lsum += psum;
      if (ragged) {
        // slots past the end may hold stale bytes (even NaN patterns): zero them so 0 * x stays 0
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (4 * g4 + i >= n_valid) {
              vv[j][i] = (__bf16)0.f;
              vv[j][4 + i] = (__bf16)0.f;
            }
      }
      const short4v bh = __builtin_bit_cast(short4v, phi);
      const short4v bl = __builtin_bit_cast(short4v, plo);
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const bf16x8 w = vv[dt >> 1];
        const bf16x4 half = (dt & 1) ? bf16x4{w[4], w[5], w[6], w[7]} : bf16x4{w[0], w[1], w[2], w[3]};
        const short4v av = __builtin_bit_cast(short4v, half);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bh, O[dt], 0, 0, 0);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bl, O[dt], 0, 0, 0);
      }
    };

    // Finished pieces are not stored to global memory right away: stores share the in-order
    // vmcnt queue with the tile loads, and a store in the middle of the stream makes the next
    // tile wait for the store's acknowledgement.  They are queued in LDS (a separate counter)
    // and written when the wave has streamed its whole range (or when the queue is full).
    float* qbase = lds + WPW * slot_floats + 2 * WPW + wv * stream_wave_queue_floats(G, a.qs, a.aq);
    const int qstride = slot_floats + 8;
    int qn = 0;
    auto flush_outputs = [&]() {
      for (int i = 0; i < qn; ++i) {
        const float* e = qbase + i * qstride;
        const int* meta = (const int*)(e + slot_floats);
        const int kind = rfl(meta[0]), r = rfl(meta[1]), g = rfl(meta[2]), gslot = rfl(meta[3]);
        if (col < G) {
          float4v o4[8];
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) o4[dt] = *(const float4v*)(e + col * 128 + 16 * dt + 4 * g4);
          const float m_e = e[G * 128 + col], l_e = e[G * 128 + G + col];
          if (kind == 0) {                                   // final: normalise and write to `out`
            const float inv = a.out_scale / l_e;
            const int64_t o_base = ((int64_t)r * a.Hq + g * G + col) * HD + 4 * g4;
            if (a.out_bf16) {
              unsigned short* o = (unsigned short*)a.out + o_base;
#pragma unroll
              for (int dt = 0; dt < HD / 16; ++dt) {
                uint2v pk;
                pk[0] = (unsigned)float_to_bf16_bits(o4[dt][0] * inv) | ((unsigned)float_to_bf16_bits(o4[dt][1] * inv) << 16);
                pk[1] = (unsigned)float_to_bf16_bits(o4[dt][2] * inv) | ((unsigned)float_to_bf16_bits(o4[dt][3] * inv) << 16);
                __builtin_nontemporal_store(pk, (uint2v*)(o + 16 * dt));
              }
            } else {
              float* o = (float*)a.out + o_base;
#pragma unroll
              for (int dt = 0; dt < HD / 16; ++dt) __builtin_nontemporal_store(o4[dt] * inv, (float4v*)(o + 16 * dt));
            }
          } else {                                           // un-normalised state to the HBM workspace
            const int64_t pi = (int64_t)gslot * a.Hq + g * G + col;
            float* o = a.part_o + pi * 128 + 4 * g4;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
              store_pair_agent(o + 16 * dt, o4[dt][0], o4[dt][1]);
              store_pair_agent(o + 16 * dt + 2, o4[dt][2], o4[dt][3]);
            }
            if (g4 == 0) store_pair_agent((float*)&a.part_ml[pi], m_e, l_e);
          }
        }
      }
      qn = 0;
    };
    auto enqueue = [&](int kind, int gslot, float l_all) {
      if (qn == a.qs) flush_outputs();
      float* e = qbase + qn * qstride;
      if (col < G) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *(float4v*)(e + col * 128 + 16 * dt + 4 * g4) = O[dt];
        if (g4 == 0) {
          e[G * 128 + col] = m;
          e[G * 128 + G + col] = l_all;
        }
      }
      if (lane == 0) {
        int* meta = (int*)(e + slot_floats);
        meta[0] = kind;
        meta[1] = cc.r;
        meta[2] = cc.g;
        meta[3] = gslot;
      }
      ++qn;
    };
    auto write_out = [&](float l_all) { enqueue(0, 0, l_all); };
    auto write_partial = [&](int gslot, float l_all) { enqueue(1, gslot, l_all); };
    auto park = [&](float l_all, bool to_end) {               // hand this wave's first piece to its left neighbour
      float* so = lds + wv * slot_floats;
      if (col < G) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *(float4v*)(so + col * 128 + 16 * dt + 4 * g4) = O[dt];
        if (g4 == 0) {
          so[G * 128 + col] = m;
          so[G * 128 + G + col] = l_all;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (lane == 0) {
        flag_set(2 * wv + 1, to_end);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        flag_set(2 * wv, 1);
      }
    };

    // The piece [.., cc.t] of segment (cc.r, cc.g) is finished.  `last` = it is the last tile of
    // this wave's range.  A piece that spans its whole segment is final; otherwise it is part
    // of a chain of pieces of neighbouring waves (see the header comment).
    auto emit = [&](bool to_end, bool last) {
      float l_all = column_sum(lsum);
      if (last && !to_end && wv < WPW - 1) {
        // the segment continues in the right-hand neighbour's range: fold its first piece in
        while (flag_get(2 * (wv + 1)) == 0) __builtin_amdgcn_s_sleep(2);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        to_end = flag_get(2 * (wv + 1) + 1) != 0;
        const float* so = lds + (wv + 1) * slot_floats;
        const int c = col < G ? col : 0;
        const float m2 = so[G * 128 + c], l2 = so[G * 128 + G + c];
        const float m_new = fmaxf(m, m2);
        const float a1 = __builtin_amdgcn_exp2f(m - m_new), a2 = __builtin_amdgcn_exp2f(m2 - m_new);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          const float4v o2 = *(const float4v*)(so + c * 128 + 16 * dt + 4 * g4);
          O[dt] = O[dt] * a1 + o2 * a2;
        }
        m = m_new;
        l_all = l_all * a1 + l2 * a2;
      }
      if (from_start && to_end) write_out(l_all);
      else if (!from_start) {
        // began before this wave's range: the left neighbour (or, for wave 0, the work-group on
        // the left through the workspace) continues the chain
        if (wv == 0) write_partial(2 * blockIdx.x, l_all);
        else park(l_all, to_end);
      } else write_partial(2 * blockIdx.x + 1, l_all);       // starts here, ends in a later work-group
    };

    // main loop: NBUF tiles per trip so that buffer indices are compile-time constants.
    // Order inside a step matters because vmcnt retires in order: the queries of the next
    // segment are requested BEFORE this step's tile loads and adopted one step later AFTER
    // that step's tile loads, so waiting for them never drains the tile pipeline.
    bool q_pending = true;                                   // the first segment's queries wait in qnext
    for (int i = 0; i < n_my; i += NBUF) {
#pragma unroll
      for (int u = 0; u < NBUF; ++u) {
        const bool active = i + u < n_my;
        const bool seg_end = active && cc.t == cc.tiles - 1;
        const bool more = i + u + 1 < n_my;
        if (q_pending && seg_end && more) {
          // a one-tile segment: its successor's queries are requested below, so the ones waiting
          // in qnext must be adopted first (this wait can stall; the common case is further down)
          adopt_q(qnext);
          q_pending = false;
        }
        if (seg_end && more) {
          const int ng = cc.g + 1 == Hkv ? 0 : cc.g + 1;
          const int nr = cc.g + 1 == Hkv ? cc.r_next : cc.r;
          load_q(qnext, nr, ng);
        }
        if (FUSED && active) {
          // fetch the appended row one tile before it is needed when the segment allows it
          if (seg_end ? !new_ready : (more && cc.t + 2 == cc.tiles)) {
            load_new(cc.r, cc.g);
            new_ready = true;
          }
        }
        issue(kb[(u + NBUF - 1) % NBUF], vb[(u + NBUF - 1) % NBUF]);
        if (p_left > 0) {
          advance(pc, wp);
          lookup_block(pc);
          --p_left;
        }
        if (q_pending) {
          // adopted after this step's tile loads were issued: waiting for the queries (requested a
          // step ago) then costs no more than waiting for the tile computed next
          adopt_q(qnext);
          q_pending = false;
        }
        if (active) {
          if (FUSED && seg_end) {
            patch_and_store(kb[u], vb[u]);
            new_ready = false;
          }
          compute(kb[u], vb[u]);
          TL_STAMP(8 + i + u);
#ifdef ODMA_DEV_TIMELINE
          if (lane == 0 && seg_end) tl_lds[wv][6] |= 1ll << (i + u);
          if (lane == 0 && qn == a.qs && (seg_end || !more)) tl_lds[wv][7] |= 1ll << (i + u);
#endif

          if (seg_end || !more) emit(seg_end, !more);
          if (more) {
            advance(cc, wc);
            if (seg_end) {
              q_pending = true;
              m = NEG_INF;
              lsum = 0.f;
#pragma unroll
              for (int k = 0; k < 8; ++k) O[k] = float4v{0.f, 0.f, 0.f, 0.f};
              from_start = true;
            }
          }
        }
      }
    }
    // the range is streamed: write what was queued
    TL_STAMP(2);
    flush_outputs();
    if (FUSED) flush_appends();
    TL_STAMP(3);
#ifdef ODMA_DEV_TIMELINE
    if (lane == 0) tl_lds[wv][5] = n_my;
#endif
  }

  // Outputs of empty requests are zeros: thread i of the grid looks after request i, i + grid size, ...
  for (int r = r_mine; r < a.n; r += gridDim.x * (64 * WPW)) {
    if ((r == r_mine ? tiles_mine : a.req_pos[r].tiles) == 0) {
      const int64_t o = (int64_t)r * a.Hq * HD;
      if (a.out_bf16) {
        uint2v* p = (uint2v*)((unsigned short*)a.out + o);
        for (int i = 0; i < a.Hq * (HD / 4); ++i) p[i] = uint2v{0u, 0u};
      } else {
        float4v* p = (float4v*)((float*)a.out + o);
        for (int i = 0; i < a.Hq * (HD / 4); ++i) p[i] = float4v{0.f, 0.f, 0.f, 0.f};
      }
    }
  }

#ifdef ODMA_DEV_TIMELINE
  auto tl_flush = [&]() {
    TL_STAMP(4);
    const int w = blockIdx.x * WPW + wv;
    if (w < 4096 && lane < TL_SLOTS) odma_dev_timeline_buf[w * TL_SLOTS + lane] = tl_lds[wv][lane];
  };
#else
  auto tl_flush = [&]() {};
#endif
  if (!a.fuse_reduce) {
    tl_flush();
    return;
  }
  // Merge of segments cut by work-group boundaries.  Every work-group a cut segment spans has by
  // now written one partial state to the workspace.  It then counts itself in at the segment's
  // counter; the work-group that arrives last sees all partials and merges them:
  //   m* = max m_i, w_i = 2^(m_i - m*), out = sum w_i O_i / sum w_i l_i.
  // Nobody waits for anybody.  Order: a wave's partial stores (write-through, agent scope) are
  // acknowledged (vmcnt 0) before the work-group barrier, the counter update comes after the
  // barrier, and the merging work-group reads the partials with agent-scope loads after it has
  // seen the full count.
  const int b = blockIdx.x;
  // a work-group whose range begins and ends on segment boundaries has written no partial and counts in nowhere:
  // its waves leave as they finish (the descriptors are the same for every wave, so all of them take this exit)
  if (rd_cut[0].n_parts == 0 && !(rd_cut[1].n_parts > 0 && rd_cut[1].b0 == b)) {
    tl_flush();
    return;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int* merges_here = flags;                                // chain hand-off flags are dead now
  if (threadIdx.x < 2) {
    const ReduceDesc rda = rd_cut[0], rdb = rd_cut[1];       // the segments cut at this work-group's two boundaries
    // thread 0 counts the work-group in at the segment cut in front of it (it holds a piece of that
    // segment), thread 1 at the segment that starts here and runs into the next work-group; both
    // counter updates travel together
    const bool second = threadIdx.x == 1;
    const int n_parts = second ? rdb.n_parts : rda.n_parts;
    const int owner = (second ? b : rda.b0) + 1;
    const bool in = second ? (rdb.n_parts > 0 && rdb.b0 == b) : rda.n_parts > 0;
    int last = 0;
    if (in) {
      const int old = __hip_atomic_fetch_add(a.arrive + owner, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last = old == n_parts - 1;
      // the last arrival leaves the counter at zero for the next launch
      if (last) __hip_atomic_store(a.arrive + owner, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    merges_here[threadIdx.x] = last;
  }
  __syncthreads();
  const bool do_a = merges_here[0] != 0, do_b = merges_here[1] != 0;
  if (!do_a && !do_b) {
    tl_flush();
    return;
  }
  for (int which = 0; which < 2; ++which) {
    if (!(which == 0 ? do_a : do_b)) continue;
    const ReduceDesc rd = rd_cut[which];
    const int n_parts = rd.n_parts, b0 = rd.b0;
    // thread -> (head, four channels); partial i of the segment sits in slot 2 (b0 + i), the first
    // one in its work-group's "starts here" slot 2 b0 + 1
    for (int idx = threadIdx.x; idx < G * 32; idx += 64 * WPW) {
      const int h = idx >> 5, d4 = idx & 31;
      auto part = [&](int i) -> int64_t { return (int64_t)(2 * (b0 + i) + (i == 0 ? 1 : 0)) * a.Hq + rd.g * G + h; };
      float m_run = -INFINITY, l_run = 0.f;
      float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
      // batch = partials whose loads are in flight together: the usual cut has two parts, a long request
      // spans tens of work-groups; loads past the last part would only repeat it, so the batch fits the count
      auto merge = [&](auto batch_tag) {
        constexpr int BATCH = decltype(batch_tag)::value;
        for (int i0 = 0; i0 < n_parts; i0 += BATCH) {
          float2 ml[BATCH];
          float4v ov[BATCH];
#pragma unroll
          for (int u = 0; u < BATCH; ++u) {
            const int64_t pi = part(min(i0 + u, n_parts - 1));
            ml[u] = load_pair_agent((const float*)&a.part_ml[pi]);
            const float2 lo = load_pair_agent(a.part_o + pi * 128 + 4 * d4);
            const float2 hi = load_pair_agent(a.part_o + pi * 128 + 4 * d4 + 2);
            ov[u] = float4v{lo.x, lo.y, hi.x, hi.y};
          }
          float m_new = m_run;
#pragma unroll
          for (int u = 0; u < BATCH; ++u)
            if (i0 + u < n_parts) m_new = fmaxf(m_new, ml[u].x);
          const float keep = __builtin_amdgcn_exp2f(m_run - m_new);
          acc *= keep;
          l_run *= keep;
#pragma unroll
          for (int u = 0; u < BATCH; ++u)
            if (i0 + u < n_parts) {
              const float w = __builtin_amdgcn_exp2f(ml[u].x - m_new);
              acc += ov[u] * w;
              l_run = fmaf(w, ml[u].y, l_run);
            }
          m_run = m_new;
        }
      };
      if (n_parts <= 2) merge(std::integral_constant<int, 2>{});
      else if (n_parts <= 8) merge(std::integral_constant<int, 8>{});
      else merge(std::integral_constant<int, STREAM_MERGE_BATCH>{});
      const float inv = a.out_scale / l_run;
      if (4 * d4 >= HD) continue;                            // head_dim 64: the upper channels are padding
      const int64_t o = ((int64_t)rd.r * a.Hq + rd.g * G + h) * HD + 4 * d4;
      if (a.out_bf16) {
        uint2v pk;
        pk[0] = (unsigned)float_to_bf16_bits(acc[0] * inv) | ((unsigned)float_to_bf16_bits(acc[1] * inv) << 16);
        pk[1] = (unsigned)float_to_bf16_bits(acc[2] * inv) | ((unsigned)float_to_bf16_bits(acc[3] * inv) << 16);
        *(uint2v*)((unsigned short*)a.out + o) = pk;
      } else {
        *(float4v*)((float*)a.out + o) = acc * inv;
      }
    }
  }
  tl_flush();
}

// ---------------------------------------------------------------------------------
// cross-work-group reduction as a launch of its own.  A segment cut by work-group boundaries left one partial per
// work-group it spans: the first in that group's "starts here" slot 2b+1, the others in slot
// 2b.  The plan kernel marks, for the boundary in front of every attention work-group, whether
// a segment straddles it and this is the first boundary inside that segment; if so the
// (boundary, head) work-group of this kernel merges all partials of the segment:  m* = max m_i, w_i = 2^(m_i - m*), out = sum w_i O_i / sum w_i l_i.
// ---------------------------------------------------------------------------------
// Merges n_parts partial states of one head, BATCH partials at a time with all their loads in
// flight at once; batches are chained with a running maximum.  Thread d owns channel d.
template <int BATCH, class PartFn>
__device__ __forceinline__ float merge_parts(const StreamArgs& a, PartFn part, int n_parts, int d) {
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int i0 = 0; i0 < n_parts; i0 += BATCH) {
    float2 ml[BATCH];
    float ov[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int64_t pi = part(min(i0 + u, n_parts - 1));
      ml[u] = a.part_ml[pi];
      ov[u] = a.part_o[pi * 128 + d];
    }
    float m_new = m_run;
#pragma unroll
    for (int u = 0; u < BATCH; ++u)
      if (i0 + u < n_parts) m_new = fmaxf(m_new, ml[u].x);
    const float keep = __builtin_amdgcn_exp2f(m_run - m_new);
    acc *= keep;
    l_run *= keep;
#pragma unroll
    for (int u = 0; u < BATCH; ++u)
      if (i0 + u < n_parts) {
        const float w = __builtin_amdgcn_exp2f(ml[u].x - m_new);
        acc = fmaf(w, ov[u], acc);
        l_run = fmaf(w, ml[u].y, l_run);
      }
    m_run = m_new;
  }
  return acc * (a.out_scale / l_run);
}

// grid: n_wg * G work-groups (boundary, head) of 128 threads (one per channel); no LDS, no
// barrier.  Used when the in-kernel merge of decode_stream_kernel is switched off.
__global__ __launch_bounds__(128) void stream_reduce_kernel(StreamArgs a, int n_wg) {
  const int G = a.G, d = threadIdx.x;
  const int b = blockIdx.x / G, h = blockIdx.x - b * G;
  const ReduceDesc rd = a.red[b];
  const int n_parts = rd.n_parts;
  if (n_parts == 0 || rd.b0 != b - 1) return;               // nothing cut here, or an earlier boundary owns the merge
  const int g = rd.g, b0 = rd.b0;
  // partial i of this segment: the first sits in its work-group's "starts here" slot
  auto part = [&](int i) -> int64_t { return (int64_t)(2 * (b0 + i) + (i == 0 ? 1 : 0)) * a.Hq + g * G + h; };
  // most cut segments span two work-groups; a long request spans tens
  const float val = n_parts <= 4 ? merge_parts<4>(a, part, n_parts, d) : merge_parts<16>(a, part, n_parts, d);
  if (d >= a.head_dim) return;                               // head_dim 64: the upper channels are padding
  const int64_t o = ((int64_t)rd.r * a.Hq + g * G + h) * a.head_dim + d;
  if (a.out_bf16) __builtin_nontemporal_store(float_to_bf16_bits(val), (unsigned short*)a.out + o);
  else __builtin_nontemporal_store(val, (float*)a.out + o);
}

}  // namespace
