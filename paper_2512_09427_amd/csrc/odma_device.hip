// Device side of libodma for gfx950 (MI355X): KV append, batched GQA decode attention
// over contiguous slabs or paged blocks, cross-split reduction, migration copy, export.
//
// Decode attention is a streaming scan of K and V with no reuse, so it is bounded by
// HBM bandwidth; the design goal is bytes in flight, not arithmetic:
//   * work item = (request, KV head, chunk of tokens); chunks have one size per call so
//     the heavy tail of the length distribution spreads over the whole chip;
//   * one wavefront owns one item at a time and keeps its online-softmax state
//     (running max m, sum l, accumulator O) in registers; waves never synchronise;
//   * the pool's block format is the matrix-core operand order, so every wave-wide load
//     is one contiguous 1 KiB run and lands directly in the registers the MFMA reads:
//     no LDS staging, no transposes;
//   * the 7 query heads of a GQA group are the columns of the MFMA B operand, so a K or V
//     byte is loaded once per group;
//   * partial (m, l, O) of multi-chunk requests go to a workspace and are merged by
//     log-sum-exp in a second kernel; single-chunk requests write their output directly.
#include <hip/hip_runtime.h>

#include <cmath>
#include <string>

#include "odma_internal.h"

namespace odma {
int migrate_begin(odma_pool* pool, int32_t rid, int64_t* new_off);
void migrate_abort(odma_pool* pool, int64_t new_off);
void migrate_commit(odma_pool* pool, int32_t rid, int64_t new_off);
}  // namespace odma

namespace {

constexpr int BLK = ODMA_BLOCK_TOKENS;
constexpr int PLAN_THREADS = 1024;
constexpr int PLAN_LDS_REQ = 8192;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

struct PlanHeader {
  int32_t n_pairs;       // number of (request, chunk) pairs
  int32_t chunk;         // tokens per chunk, multiple of 64
  int32_t n_req;
  int32_t pad;
  int64_t total_tokens;
};
struct Item {            // one (request, chunk) pair; replicated over KV heads by the kernels
  int32_t r, tok_start, n_tok, n_split;
};
struct ReqInfo {
  int32_t first_pair, n_split;
};

struct DecodeArgs {
  const char* k;         // layer base of the K pool
  const char* v;
  const void* q;
  void* out;
  const int64_t* offsets;
  const int32_t* lengths;
  const int32_t* bt;
  int32_t bt_stride;
  const PlanHeader* hdr;
  const Item* items;
  const ReqInfo* req;
  float2* part_ml;
  float* part_o;
  int32_t n, Hq, Hkv, G, D;
  int64_t head_stride;   // bytes between KV-head planes of one layer
  float scale_log2;      // sm_scale * log2(e)
  int32_t out_bf16;
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __uint_as_float((unsigned int)b << 16);
}
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
  __bf16 h = (__bf16)f;   // round to nearest even (v_cvt_pk_bf16_f32)
  return __builtin_bit_cast(unsigned short, h);
}

// ---------------------------------------------------------------------------------
// plan: lengths -> chunk size, per-request split counts, list of (request, chunk) pairs
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(PLAN_THREADS) void plan_kernel(const int32_t* __restrict__ lengths, int32_t n,
                                                            int32_t target_pairs, int32_t min_chunk,
                                                            int32_t max_pairs, PlanHeader* hdr,
                                                            ReqInfo* req_info, Item* items) {
  __shared__ long long red[PLAN_THREADS / 64];
  __shared__ int wave_tot[PLAN_THREADS / 64];
  __shared__ int first_lds[PLAN_LDS_REQ];
  __shared__ int s_chunk;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

  // total tokens
  long long t = 0;
  for (int r = tid; r < n; r += PLAN_THREADS) t += max(lengths[r], 0);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) t += __shfl_xor(t, o);
  if (lane == 0) red[wv] = t;
  __syncthreads();
  if (tid == 0) {
    long long tot = 0;
    for (int i = 0; i < PLAN_THREADS / 64; ++i) tot += red[i];
    // one chunk size for the whole call: about target_pairs equal pieces, never so many
    // that the work list outgrows the workspace (sum ceil(len/C) <= T/C + n)
    long long budget = min((long long)target_pairs, (long long)(max_pairs - n));
    if (budget < 1) budget = 1;
    long long c = (tot + budget - 1) / budget;
    c = (c + 63) / 64 * 64;
    if (c < min_chunk) c = min_chunk;
    if (c > (1 << 30)) c = 1 << 30;
    s_chunk = (int)c;
    hdr->chunk = (int)c;
    hdr->n_req = n;
    hdr->total_tokens = tot;
  }
  __syncthreads();
  const int chunk = s_chunk;

  // exclusive scan of split counts; thread t owns requests [t*per, (t+1)*per)
  const int per = (n + PLAN_THREADS - 1) / PLAN_THREADS;
  const int r0 = min(tid * per, n), r1 = min(r0 + per, n);
  int local = 0;
  for (int r = r0; r < r1; ++r) local += (max(lengths[r], 0) + chunk - 1) / chunk;
  int incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int y = __shfl_up(incl, o);
    if (lane >= o) incl += y;
  }
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < wv; ++i) base += wave_tot[i];
  int run = base + incl - local;
  const bool use_lds = n <= PLAN_LDS_REQ;
  for (int r = r0; r < r1; ++r) {
    int ns = (max(lengths[r], 0) + chunk - 1) / chunk;
    req_info[r] = ReqInfo{run, ns};
    if (use_lds) first_lds[r] = run;
    run += ns;
  }
  int n_pairs = 0;
  for (int i = 0; i < PLAN_THREADS / 64; ++i) n_pairs += wave_tot[i];
  if (tid == 0) hdr->n_pairs = n_pairs;
  __threadfence_block();
  __syncthreads();

  // pair p belongs to the last request whose first_pair <= p and that has splits
  for (int p = tid; p < n_pairs; p += PLAN_THREADS) {
    int lo = 0, hi = n - 1;            // find largest r with first[r] <= p
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      int f = use_lds ? first_lds[mid] : req_info[mid].first_pair;
      if (f <= p) lo = mid; else hi = mid - 1;
    }
    // empty requests share first_pair with their successor, so the largest r with
    // first[r] <= p is always the request that owns pair p
    int f = use_lds ? first_lds[lo] : req_info[lo].first_pair;
    int len = max(lengths[lo], 0);
    int ns = (len + chunk - 1) / chunk;
    int c = p - f;
    Item itx;
    itx.r = lo;
    itx.tok_start = c * chunk;
    itx.n_tok = min(chunk, len - c * chunk);
    itx.n_split = ns;
    items[p] = itx;
  }
}

// ---------------------------------------------------------------------------------
// shared tail: write a wave's result for (pair p, head h)
// ---------------------------------------------------------------------------------

// ---------------------------------------------------------------------------------
// MFMA decode kernel: bf16 storage, D = 128, G <= 16.
//   S^T[16 tok x 16 heads] = K_blk[16 x 128] * Q^T[128 x 16]      4 x mfma 16x16x32
//   O^T[128 d x 16 heads] += V_blk^T[128 x 16 tok] * P^T[16 x 16]  8 x mfma 16x16x16 (x2: hi/lo)
// Lane l: column (head) l%16 of S^T, P^T, O^T; rows 4*(l/16)..+3.  The running max, the sum
// and the rescale factor of a head therefore live in the lanes that hold its columns.
// P is split into bf16 hi + lo parts so the P*V product keeps ~16 bits of P.
// ---------------------------------------------------------------------------------
template <bool PAGED>
__global__ __launch_bounds__(256, 2) void decode_mfma_kernel(DecodeArgs a) {
  const int lane = threadIdx.x & 63;
  const int head = lane & 15, g4 = lane >> 4;
  const int n_waves = gridDim.x * 4;
  const int wave_id = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n_items = a.hdr->n_pairs * a.Hkv;
  constexpr int BLOCK_BYTES = BLK * 128 * 2;
  const float NEG_INF = -INFINITY;

  for (int it = wave_id; it < n_items; it += n_waves) {
    const int p = it / a.Hkv, g = it - p * a.Hkv;
    const Item item = a.items[p];
    const int r = item.r, n_tok = item.n_tok;
    const int n_blk = (n_tok + BLK - 1) / BLK;            // blocks this item touches
    const int blk_first = item.tok_start / BLK;           // logical block index in the request
    const char* kplane = a.k + (int64_t)g * a.head_stride + lane * 16;
    const char* vplane = a.v + (int64_t)g * a.head_stride + lane * 16;
    int64_t slab_blk = 0;
    const int32_t* bt_row = nullptr;
    if (PAGED) bt_row = a.bt + (int64_t)r * a.bt_stride + blk_first;
    else slab_blk = a.offsets[r] / BLK + blk_first;

    // Q^T operand: lane (head, g4) holds q[head][32 j + 8 g4 .. +8] for the four k-steps
    bf16x8 qreg[4];
    {
      const bf16x8* qp = (const bf16x8*)((const unsigned short*)a.q + ((int64_t)r * a.Hq + g * a.G + head) * 128 + 8 * g4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        qreg[j] = head < a.G ? qp[4 * j] : z;
      }
    }

    float m = NEG_INF, lsum = 0.f;
    float4v O[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) O[i] = float4v{0.f, 0.f, 0.f, 0.f};

    const int n_tiles = (n_tok + 31) / 32;
    bf16x8 kA[2][4], vA[2][4], kB[2][4], vB[2][4];

    auto phys = [&](int b) -> int64_t {                    // physical block of the item's b-th block
      b = min(b, n_blk - 1);
      if (PAGED) return (int64_t)bt_row[b];
      return slab_blk + b;
    };
    auto load_tile = [&](int t, bf16x8 (&kk)[2][4], bf16x8 (&vv)[2][4]) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int64_t pb = phys(2 * t + h) * BLOCK_BYTES;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          kk[h][j] = *(const bf16x8*)(kplane + pb + j * 1024);
          vv[h][j] = *(const bf16x8*)(vplane + pb + j * 1024);
        }
      }
    };
    auto compute_tile = [&](int t, bf16x8 (&kk)[2][4], bf16x8 (&vv)[2][4]) {
      float4v s[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        s[h] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) s[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kk[h][j], qreg[j], s[h], 0, 0, 0);
      }
      const int tok0 = t * 32 + 4 * g4;                    // item-relative token of s[0][0]
      const bool tail = (t * 32 + 32 > n_tok);
      float x[2][4];
      float tmax = NEG_INF;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float val = s[h][i] * a.scale_log2;
          if (tail && tok0 + 16 * h + i >= n_tok) val = NEG_INF;
          x[h][i] = val;
          tmax = fmaxf(tmax, val);
        }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      m = m_new;
      float psum = 0.f;
      bf16x4 phi[2], plo[2];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float pv = __builtin_amdgcn_exp2f(x[h][i] - m_new);
          psum += pv;
          __bf16 hi = (__bf16)pv;
          phi[h][i] = hi;
          plo[h][i] = (__bf16)(pv - (float)hi);
        }
      lsum = lsum * alpha + psum;
#pragma unroll
      for (int i = 0; i < 8; ++i) O[i] *= alpha;
      if (tail) {
        // slots past the end may hold stale bytes (even NaN patterns): zero them so 0 * x stays 0
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (tok0 + 16 * h + i >= n_tok) {
                vv[h][j][i] = (__bf16)0.f;
                vv[h][j][4 + i] = (__bf16)0.f;
              }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const short4v bh = __builtin_bit_cast(short4v, phi[h]);
        const short4v bl = __builtin_bit_cast(short4v, plo[h]);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          bf16x8 w = vv[h][dt >> 1];
          bf16x4 half = (dt & 1) ? bf16x4{w[4], w[5], w[6], w[7]} : bf16x4{w[0], w[1], w[2], w[3]};
          const short4v av = __builtin_bit_cast(short4v, half);
          O[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bh, O[dt], 0, 0, 0);
          O[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bl, O[dt], 0, 0, 0);
        }
      }
    };

    if (n_tiles > 0) load_tile(0, kA, vA);
    for (int t = 0; t < n_tiles; t += 2) {
      if (t + 1 < n_tiles) load_tile(t + 1, kB, vB);
      compute_tile(t, kA, vA);
      if (t + 1 < n_tiles) {
        if (t + 2 < n_tiles) load_tile(t + 2, kA, vA);
        compute_tile(t + 1, kB, vB);
      }
    }

    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (head < a.G) {
      const int h_abs = g * a.G + head;
      if (item.n_split == 1) {
        const float inv = 1.0f / lsum;
        const int64_t o_base = ((int64_t)r * a.Hq + h_abs) * 128 + 4 * g4;
        if (a.out_bf16) {
          unsigned short* o = (unsigned short*)a.out + o_base;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) {
            uint2v pk;
            pk[0] = (unsigned)float_to_bf16_bits(O[dt][0] * inv) | ((unsigned)float_to_bf16_bits(O[dt][1] * inv) << 16);
            pk[1] = (unsigned)float_to_bf16_bits(O[dt][2] * inv) | ((unsigned)float_to_bf16_bits(O[dt][3] * inv) << 16);
            *(uint2v*)(o + 16 * dt) = pk;
          }
        } else {
          float* o = (float*)a.out + o_base;
#pragma unroll
          for (int dt = 0; dt < 8; ++dt) *(float4v*)(o + 16 * dt) = O[dt] * inv;
        }
      } else {
        float* o = a.part_o + ((int64_t)p * a.Hq + h_abs) * 128 + 4 * g4;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *(float4v*)(o + 16 * dt) = O[dt];
        if (g4 == 0) a.part_ml[(int64_t)p * a.Hq + h_abs] = make_float2(m, lsum);
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// VALU decode kernel: any storage dtype, D % 32 == 0 (<= 256), G <= 16.  One 64-lane
// work-group per item.  Scores: lane = token (64-token tiles); P*V: lane = channel.
// ---------------------------------------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<unsigned short> {
  static constexpr int X = 8;   // elements per 16 bytes
  static __device__ __forceinline__ float widen(unsigned short v) { return bf16_bits_to_float(v); }
};
template <> struct Elem<float> {
  static constexpr int X = 4;
  static __device__ __forceinline__ float widen(float v) { return v; }
};

template <typename T, bool PAGED>
__global__ __launch_bounds__(64) void decode_valu_kernel(DecodeArgs a) {
  constexpr int X = Elem<T>::X;
  constexpr int GMAX = 16, KMAX = 4;                       // heads per group, channels per lane
  __shared__ float q_lds[GMAX * 256];
  __shared__ float p_lds[GMAX * 64];
  const int lane = threadIdx.x;
  const int D = a.D, G = a.G;
  const int n_items = a.hdr->n_pairs * a.Hkv;
  const int64_t block_elems = (int64_t)BLK * D;
  const float NEG_INF = -INFINITY;

  for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
    const int p = it / a.Hkv, g = it - p * a.Hkv;
    const Item item = a.items[p];
    const int r = item.r, n_tok = item.n_tok;
    const int n_blk = (n_tok + BLK - 1) / BLK;
    const int blk_first = item.tok_start / BLK;
    const T* kplane = (const T*)(a.k + (int64_t)g * a.head_stride);
    const T* vplane = (const T*)(a.v + (int64_t)g * a.head_stride);
    const int32_t* bt_row = PAGED ? a.bt + (int64_t)r * a.bt_stride + blk_first : nullptr;
    const int64_t slab_blk = PAGED ? 0 : a.offsets[r] / BLK + blk_first;
    auto phys = [&](int b) -> int64_t {
      b = min(b, n_blk - 1);
      return PAGED ? (int64_t)bt_row[b] : slab_blk + b;
    };

    __syncthreads();                                        // previous item done with LDS
    {
      const T* qp = (const T*)a.q + ((int64_t)r * a.Hq + g * G) * D;
      for (int i = lane; i < G * D; i += 64) q_lds[(i / D) * 256 + i % D] = Elem<T>::widen(qp[i]);
    }
    __syncthreads();

    float m[GMAX], lsum[GMAX], o[GMAX][KMAX];
#pragma unroll
    for (int h = 0; h < GMAX; ++h) {
      m[h] = NEG_INF;
      lsum[h] = 0.f;
#pragma unroll
      for (int k = 0; k < KMAX; ++k) o[h][k] = 0.f;
    }

    const int n_tiles = (n_tok + 63) / 64;
    for (int t = 0; t < n_tiles; ++t) {
      // ---- scores: this lane's token against G queries
      const int tok = t * 64 + lane;
      const T* kb = kplane + phys(4 * t + (lane >> 4)) * block_elems + (lane & 15) * X;
      float s[GMAX];
#pragma unroll
      for (int h = 0; h < GMAX; ++h) s[h] = 0.f;
      for (int dc = 0; dc < D / X; ++dc) {
        float kv[X];
        if (X == 8) {
          uint4v raw = *(const uint4v*)(kb + (int64_t)dc * BLK * X);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            kv[2 * i] = __uint_as_float(raw[i] << 16);
            kv[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
          }
        } else {
          float4v raw = *(const float4v*)(kb + (int64_t)dc * BLK * X);
#pragma unroll
          for (int i = 0; i < 4; ++i) kv[i] = raw[i];
        }
#pragma unroll
        for (int h = 0; h < GMAX; ++h)
          if (h < G) {
            const float* qh = q_lds + h * 256 + dc * X;
#pragma unroll
            for (int i = 0; i < X; ++i) s[h] = fmaf(qh[i], kv[i], s[h]);
          }
      }
      // ---- online softmax per head (base 2)
      __syncthreads();                                      // p_lds free again
#pragma unroll
      for (int h = 0; h < GMAX; ++h)
        if (h < G) {
          float x = tok < n_tok ? s[h] * a.scale_log2 : NEG_INF;
          float m_new = fmaxf(m[h], wave_max(x));
          float alpha = __builtin_amdgcn_exp2f(m[h] - m_new);
          float pv = __builtin_amdgcn_exp2f(x - m_new);
          m[h] = m_new;
          lsum[h] = lsum[h] * alpha + pv;
#pragma unroll
          for (int k = 0; k < KMAX; ++k) o[h][k] *= alpha;
          p_lds[h * 64 + lane] = pv;
        }
      __syncthreads();
      // ---- P*V: this lane's channels d = lane + 64 k
      const int nb_tile = min(4, n_blk - 4 * t);
      for (int b = 0; b < nb_tile; ++b) {
        const T* vb = vplane + phys(4 * t + b) * block_elems;
        const int t_valid = min(BLK, n_tok - (t * 64 + b * BLK));   // tokens of this block in range
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
          const int d = lane + 64 * k;
          if (d < D) {
            float vals[BLK];
            const T* vrow = vb + ((int64_t)(d >> 5) * 4 * 16 + (d & 15)) * 8 + ((d >> 4) & 1) * 4;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
              const T* src = vrow + t4 * 16 * 8;
              if (X == 8) {
                uint2v raw = *(const uint2v*)src;
                vals[4 * t4 + 0] = __uint_as_float(raw[0] << 16);
                vals[4 * t4 + 1] = __uint_as_float(raw[0] & 0xffff0000u);
                vals[4 * t4 + 2] = __uint_as_float(raw[1] << 16);
                vals[4 * t4 + 3] = __uint_as_float(raw[1] & 0xffff0000u);
              } else {
                float4v raw = *(const float4v*)src;
#pragma unroll
                for (int i = 0; i < 4; ++i) vals[4 * t4 + i] = raw[i];
              }
            }
            // stale slots past the end may hold anything: keep 0 * x == 0
#pragma unroll
            for (int i = 0; i < BLK; ++i)
              if (i >= t_valid) vals[i] = 0.f;
#pragma unroll
            for (int h = 0; h < GMAX; ++h)
              if (h < G) {
                const float* ph = p_lds + h * 64 + b * BLK;
                float acc = o[h][k];
#pragma unroll
                for (int i = 0; i < BLK; ++i) acc = fmaf(ph[i], vals[i], acc);
                o[h][k] = acc;
              }
          }
        }
      }
    }

    // ---- result
#pragma unroll
    for (int h = 0; h < GMAX; ++h)
      if (h < G) {
        const float l_tot = wave_sum(lsum[h]);
        const int h_abs = g * G + h;
        if (item.n_split == 1) {
          const float inv = 1.0f / l_tot;
#pragma unroll
          for (int k = 0; k < KMAX; ++k) {
            const int d = lane + 64 * k;
            if (d < D) {
              const int64_t idx = ((int64_t)r * a.Hq + h_abs) * D + d;
              if (a.out_bf16) ((unsigned short*)a.out)[idx] = float_to_bf16_bits(o[h][k] * inv);
              else ((float*)a.out)[idx] = o[h][k] * inv;
            }
          }
        } else {
#pragma unroll
          for (int k = 0; k < KMAX; ++k) {
            const int d = lane + 64 * k;
            if (d < D) a.part_o[((int64_t)p * a.Hq + h_abs) * D + d] = o[h][k];
          }
          if (lane == 0) a.part_ml[(int64_t)p * a.Hq + h_abs] = make_float2(m[h], l_tot);
        }
      }
  }
}

// ---------------------------------------------------------------------------------
// cross-split reduction: one wave per (request, query head)
//   m* = max m_i, w_i = 2^(m_i - m*), out = sum w_i o_i / sum w_i l_i
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void reduce_kernel(DecodeArgs a) {
  const int lane = threadIdx.x & 63;
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= a.n * a.Hq) return;
  const int r = w / a.Hq, h = w - r * a.Hq;
  const ReqInfo info = a.req[r];
  if (info.n_split == 1) return;                            // written by the attention kernel
  const int D = a.D;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  float l_star = 1.f;
  if (info.n_split > 1) {
    float m_star = -INFINITY;
    for (int i = lane; i < info.n_split; i += 64)
      m_star = fmaxf(m_star, a.part_ml[(int64_t)(info.first_pair + i) * a.Hq + h].x);
    m_star = wave_max(m_star);
    l_star = 0.f;
    for (int i = 0; i < info.n_split; ++i) {
      const int64_t pi = (int64_t)(info.first_pair + i) * a.Hq + h;
      const float2 ml = a.part_ml[pi];
      const float wgt = __builtin_amdgcn_exp2f(ml.x - m_star);
      l_star = fmaf(wgt, ml.y, l_star);
      const float* po = a.part_o + pi * D;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int d = lane + 64 * k;
        if (d < D) acc[k] = fmaf(wgt, po[d], acc[k]);
      }
    }
  }
  const float inv = 1.0f / l_star;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int d = lane + 64 * k;
    if (d < D) {
      const int64_t idx = ((int64_t)r * a.Hq + h) * D + d;
      if (a.out_bf16) ((unsigned short*)a.out)[idx] = float_to_bf16_bits(acc[k] * inv);
      else ((float*)a.out)[idx] = acc[k] * inv;
    }
  }
}

// ---------------------------------------------------------------------------------
// append / export: row-major rows <-> pool block format
// ---------------------------------------------------------------------------------
struct RowArgs {
  char* k;               // layer base
  char* v;
  int64_t head_stride;   // bytes
  int32_t Hkv, D;
};

// element index inside a block
__device__ __forceinline__ int k_index(int t, int d, int X) { return ((d / X) * BLK + t) * X + d % X; }
__device__ __forceinline__ int v_index(int t, int d) {
  return (((d >> 5) * 4 + (t >> 2)) * 16 + (d & 15)) * 8 + ((d >> 4) & 1) * 4 + (t & 3);
}

template <typename T>
__global__ __launch_bounds__(256) void append_kernel(RowArgs a, int32_t n, const int64_t* __restrict__ offsets,
                                                     const int32_t* __restrict__ positions,
                                                     const int32_t* __restrict__ n_new,
                                                     const int64_t* __restrict__ src_start,
                                                     const int32_t* __restrict__ bt, int32_t bt_stride,
                                                     const T* __restrict__ k_new, const T* __restrict__ v_new) {
  constexpr int X = 16 / sizeof(T);
  const int r = blockIdx.y;
  const int cnt = n_new ? n_new[r] : 1;
  const int j0 = blockIdx.x * BLK;
  if (j0 >= cnt) return;
  const int j1 = min(j0 + BLK, cnt);
  const int64_t src0 = src_start ? src_start[r] : (int64_t)r;
  const int pos0 = positions[r];
  const int row_elems = a.Hkv * a.D;
  const int chunks = row_elems / X;
  const int64_t block_elems = (int64_t)BLK * a.D;
  for (int j = j0; j < j1; ++j) {
    const int pos = pos0 + j;
    const int64_t blk = bt ? (int64_t)bt[(int64_t)r * bt_stride + pos / BLK] : offsets[r] / BLK + pos / BLK;
    const int t = pos % BLK;
    const T* ks = k_new + (src0 + j) * row_elems;
    const T* vs = v_new + (src0 + j) * row_elems;
    for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
      const int e0 = c * X, g = e0 / a.D, d0 = e0 % a.D;
      T* kd = (T*)(a.k + (int64_t)g * a.head_stride) + blk * block_elems;
      T* vd = (T*)(a.v + (int64_t)g * a.head_stride) + blk * block_elems;
      *(uint4v*)(kd + k_index(t, d0, X)) = *(const uint4v*)(ks + e0);
      alignas(16) T tmp[X];
      *(uint4v*)tmp = *(const uint4v*)(vs + e0);
#pragma unroll
      for (int i = 0; i < X; ++i) vd[v_index(t, d0 + i)] = tmp[i];
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(RowArgs a, int64_t offset, int32_t length,
                                                     const int32_t* __restrict__ block_row,
                                                     T* __restrict__ k_out, T* __restrict__ v_out) {
  constexpr int X = 16 / sizeof(T);
  const int row_elems = a.Hkv * a.D;
  const int chunks = row_elems / X;
  const int64_t block_elems = (int64_t)BLK * a.D;
  for (int pos = blockIdx.x; pos < length; pos += gridDim.x) {
    const int64_t blk = block_row ? (int64_t)block_row[pos / BLK] : offset / BLK + pos / BLK;
    const int t = pos % BLK;
    for (int c = threadIdx.x; c < chunks; c += blockDim.x) {
      const int e0 = c * X, g = e0 / a.D, d0 = e0 % a.D;
      const T* kd = (const T*)(a.k + (int64_t)g * a.head_stride) + blk * block_elems;
      const T* vd = (const T*)(a.v + (int64_t)g * a.head_stride) + blk * block_elems;
      *(uint4v*)(k_out + (int64_t)pos * row_elems + e0) = *(const uint4v*)(kd + k_index(t, d0, X));
      alignas(16) T tmp[X];
#pragma unroll
      for (int i = 0; i < X; ++i) tmp[i] = vd[v_index(t, d0 + i)];
      *(uint4v*)(v_out + (int64_t)pos * row_elems + e0) = *(uint4v*)tmp;
    }
  }
}

// ---------------------------------------------------------------------------------
// migration copy: for every (layer, KV head, K|V) one linear run of whole blocks
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void migrate_copy_kernel(char* k_pool, char* v_pool, int64_t plane_stride,
                                                           int64_t src_byte, int64_t dst_byte, int64_t n_bytes) {
  // blockIdx.y = plane (layer * Hkv + head) * 2 + {0: K, 1: V}
  const int plane = blockIdx.y >> 1;
  char* base = ((blockIdx.y & 1) ? v_pool : k_pool) + (int64_t)plane * plane_stride;
  const uint4v* src = (const uint4v*)(base + src_byte);
  uint4v* dst = (uint4v*)(base + dst_byte);
  const int64_t n16 = n_bytes / 16;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// ---------------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------------
int hip_fail(const char* where, hipError_t e) {
  odma::set_error(std::string(where) + ": " + hipGetErrorString(e));
  return ODMA_HIP_ERROR;
}

int device_ready(odma_pool* pool, const char* where) {
  if (!pool) {
    odma::set_error(std::string(where) + ": null pool");
    return ODMA_INVALID_ARG;
  }
  if (!pool->cfg.k_pool || !pool->cfg.v_pool) {
    odma::set_error(std::string(where) + ": pool was created without device memory");
    return ODMA_INVALID_ARG;
  }
  if (pool->n_cu == 0) {
    int dev = 0, cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(where, e);
    e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(where, e);
    pool->n_cu = cu > 0 ? cu : 256;
  }
  return ODMA_OK;
}

RowArgs row_args(const odma_pool* pool, int32_t layer) {
  RowArgs a;
  const int64_t head_stride = pool->pool_blocks * BLK * pool->cfg.head_dim * (int64_t)pool->elem_bytes;
  const int64_t layer_stride = head_stride * pool->cfg.n_kv_heads;
  a.k = (char*)pool->cfg.k_pool + layer * layer_stride;
  a.v = (char*)pool->cfg.v_pool + layer * layer_stride;
  a.head_stride = head_stride;
  a.Hkv = pool->cfg.n_kv_heads;
  a.D = pool->cfg.head_dim;
  return a;
}

}  // namespace

extern "C" {

int odma_append_kv(odma_pool_t* pool, int32_t layer, int32_t n, const int64_t* offsets,
                   const int32_t* positions, const int32_t* n_new, const int64_t* src_start,
                   int32_t max_new, const int32_t* block_table, int32_t bt_stride, const void* k_new,
                   const void* v_new, void* stream) {
  int rc = device_ready(pool, "odma_append_kv");
  if (rc) return rc;
  if (n == 0) return ODMA_OK;
  if (layer < 0 || layer >= pool->cfg.n_layers || n < 0 || !positions || !k_new || !v_new ||
      (!block_table && !offsets) || (block_table && bt_stride <= 0) || (n_new && !src_start) || max_new < 1 ||
      (!n_new && max_new != 1)) {
    odma::set_error("odma_append_kv: invalid argument");
    return ODMA_INVALID_ARG;
  }
  RowArgs a = row_args(pool, layer);
  dim3 grid((max_new + BLK - 1) / BLK, n);
  hipStream_t s = (hipStream_t)stream;
  if (pool->elem_bytes == 2)
    hipLaunchKernelGGL(append_kernel<unsigned short>, grid, dim3(256), 0, s, a, n, offsets, positions, n_new, src_start,
                       block_table, bt_stride, (const unsigned short*)k_new, (const unsigned short*)v_new);
  else
    hipLaunchKernelGGL(append_kernel<float>, grid, dim3(256), 0, s, a, n, offsets, positions, n_new, src_start,
                       block_table, bt_stride, (const float*)k_new, (const float*)v_new);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_append_kv", e);
  return ODMA_OK;
}

int odma_gather_kv(odma_pool_t* pool, int32_t layer, int64_t offset, int32_t length, const int32_t* block_row,
                   void* k_out, void* v_out, void* stream) {
  int rc = device_ready(pool, "odma_gather_kv");
  if (rc) return rc;
  if (length == 0) return ODMA_OK;
  const int64_t pool_tokens = pool->pool_blocks * BLK;
  if (layer < 0 || layer >= pool->cfg.n_layers || length < 0 || !k_out || !v_out ||
      (!block_row && (offset < 0 || offset % BLK || offset + length > pool_tokens))) {
    odma::set_error("odma_gather_kv: invalid argument");
    return ODMA_INVALID_ARG;
  }
  RowArgs a = row_args(pool, layer);
  dim3 grid(length < 4096 ? length : 4096);
  hipStream_t s = (hipStream_t)stream;
  if (pool->elem_bytes == 2)
    hipLaunchKernelGGL(gather_kernel<unsigned short>, grid, dim3(256), 0, s, a, offset, length, block_row,
                       (unsigned short*)k_out, (unsigned short*)v_out);
  else
    hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(256), 0, s, a, offset, length, block_row, (float*)k_out,
                       (float*)v_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_gather_kv", e);
  return ODMA_OK;
}

int odma_decode_attention(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const int64_t* offsets,
                          const int32_t* lengths, const int32_t* block_table, int32_t bt_stride, void* out,
                          uint32_t flags, void* stream) {
  int rc = device_ready(pool, "odma_decode_attention");
  if (rc) return rc;
  if (n == 0) return ODMA_OK;
  const odma_pool_config_t& c = pool->cfg;
  if (!c.workspace) {
    odma::set_error("odma_decode_attention: pool has no workspace");
    return ODMA_INVALID_ARG;
  }
  if (layer < 0 || layer >= c.n_layers || n < 0 || n > c.max_requests || !q || !lengths || !out ||
      (!block_table && !offsets) || (block_table && bt_stride <= 0)) {
    odma::set_error("odma_decode_attention: invalid argument");
    return ODMA_INVALID_ARG;
  }
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)c.workspace;
  RowArgs ra = row_args(pool, layer);
  DecodeArgs a;
  a.k = ra.k;
  a.v = ra.v;
  a.q = q;
  a.out = out;
  a.offsets = offsets;
  a.lengths = lengths;
  a.bt = block_table;
  a.bt_stride = bt_stride;
  a.hdr = (const PlanHeader*)(ws + pool->ws.header);
  a.items = (const Item*)(ws + pool->ws.items);
  a.req = (const ReqInfo*)(ws + pool->ws.req_info);
  a.part_ml = (float2*)(ws + pool->ws.part_ml);
  a.part_o = (float*)(ws + pool->ws.part_o);
  a.n = n;
  a.Hq = c.n_q_heads;
  a.Hkv = c.n_kv_heads;
  a.G = c.n_q_heads / c.n_kv_heads;
  a.D = c.head_dim;
  a.head_stride = ra.head_stride;
  a.scale_log2 = c.sm_scale * 1.4426950408889634f;
  a.out_bf16 = c.out_dtype == ODMA_BF16;

  const bool mfma = pool->decode_kernel == ODMA_KERNEL_MFMA;
  // resident waves: MFMA kernel 2 work-groups of 4 waves per CU, VALU kernel 8 single-wave groups
  const int waves = pool->n_cu * 8;
  if (!(flags & ODMA_REUSE_PLAN)) {
    const int target_pairs = (2 * waves + c.n_kv_heads - 1) / c.n_kv_heads;
    const int min_chunk = mfma ? 128 : 64;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, lengths, n, target_pairs, min_chunk,
                       (int32_t)pool->ws.max_pairs, (PlanHeader*)(ws + pool->ws.header),
                       (ReqInfo*)(ws + pool->ws.req_info), (Item*)(ws + pool->ws.items));
  }
  if (mfma) {
    dim3 grid(waves / 4);
    if (block_table) hipLaunchKernelGGL(decode_mfma_kernel<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(decode_mfma_kernel<false>, grid, dim3(256), 0, s, a);
  } else {
    dim3 grid(waves);
    if (pool->elem_bytes == 2) {
      if (block_table) hipLaunchKernelGGL((decode_valu_kernel<unsigned short, true>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((decode_valu_kernel<unsigned short, false>), grid, dim3(64), 0, s, a);
    } else {
      if (block_table) hipLaunchKernelGGL((decode_valu_kernel<float, true>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((decode_valu_kernel<float, false>), grid, dim3(64), 0, s, a);
    }
  }
  hipLaunchKernelGGL(reduce_kernel, dim3((n * c.n_q_heads + 3) / 4), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_decode_attention", e);
  return ODMA_OK;
}

int odma_migrate(odma_pool_t* pool, int32_t req_id, void* stream, int64_t* new_offset, int32_t* new_cap) {
  if (!pool) {
    odma::set_error("odma_migrate: null pool");
    return ODMA_INVALID_ARG;
  }
  int64_t new_off = -1;
  int rc = odma::migrate_begin(pool, req_id, &new_off);
  if (rc) return rc;
  const odma::Request& r = pool->req[req_id];
  if (pool->cfg.k_pool && pool->cfg.v_pool && r.len > 0) {
    // one sequential copy per (layer, KV head, K|V): whole blocks covering len tokens
    const int64_t block_bytes = (int64_t)BLK * pool->cfg.head_dim * pool->elem_bytes;
    const int64_t n_bytes = (int64_t)((r.len + BLK - 1) / BLK) * block_bytes;
    const int64_t plane_stride = pool->pool_blocks * block_bytes;
    const int planes = pool->cfg.n_layers * pool->cfg.n_kv_heads;
    int64_t per_block_bytes = 256 * 16 * 8;
    int gx = (int)((n_bytes + per_block_bytes - 1) / per_block_bytes);
    if (gx < 1) gx = 1;
    if (gx > 1024) gx = 1024;
    hipLaunchKernelGGL(migrate_copy_kernel, dim3(gx, planes * 2), dim3(256), 0, (hipStream_t)stream,
                       (char*)pool->cfg.k_pool, (char*)pool->cfg.v_pool, plane_stride, (r.off / BLK) * block_bytes,
                       (new_off / BLK) * block_bytes, n_bytes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
      odma::migrate_abort(pool, new_off);
      return hip_fail("odma_migrate", e);
    }
  }
  odma::migrate_commit(pool, req_id, new_off);
  if (new_offset) *new_offset = new_off;
  if (new_cap) *new_cap = pool->cfg.large_cap;
  return ODMA_OK;
}

}  // extern "C"
