// Chunked work list (plan), the fp32 vector-ALU decode kernel and its cross-split reduction.
#pragma once

#include "kernels_common.h"

namespace {

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
    // 8 splits at a time with all their loads in flight: a long request has hundreds of splits
    constexpr int RB = 8;
    for (int i0 = 0; i0 < info.n_split; i0 += RB) {
      float2 ml[RB];
      float po[RB][4];
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int64_t pi = (int64_t)(info.first_pair + min(i0 + u, info.n_split - 1)) * a.Hq + h;
        ml[u] = a.part_ml[pi];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int d = lane + 64 * k;
          po[u][k] = d < D ? a.part_o[pi * D + d] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < RB; ++u)
        if (i0 + u < info.n_split) {
          const float wgt = __builtin_amdgcn_exp2f(ml[u].x - m_star);
          l_star = fmaf(wgt, ml[u].y, l_star);
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[k] = fmaf(wgt, po[u][k], acc[k]);
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

}  // namespace
