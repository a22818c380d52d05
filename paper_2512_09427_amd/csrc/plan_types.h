// Plain data types of the decode plans, the arithmetic that cuts the tile stream into per-wave ranges, and the
// carve-up of the device workspace.  No HIP in here: the host allocator (built with g++ alone) and the kernels
// (hipcc) both include it, so that the host can size and check what the device fills in.
#pragma once

#include <cstddef>
#include <cstdint>

#ifdef __HIPCC__
#define ODMA_HD __host__ __device__
#else
#define ODMA_HD
#endif

namespace odma_plan {

// ---- chunked scheme (vector-ALU kernel) ----
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

// ---- tile-stream scheme (matrix-core kernel) ----
struct StreamEntry {         // one non-empty request, in batch order
  int32_t r, tiles, first_pos, len;   // tiles = ceil(len/16) per KV head; first_pos = position of (r, head 0, block 0)
  int32_t base_block, pad0, pad1, pad2;
};
struct WaveDesc {            // one wave's tile range, with its first entry inlined so that the
  int32_t pos_start, pos_end, entry0, n_entries;   // first loads need no second lookup
  int32_t r, tiles, first_pos, len;
  int32_t base_block, r_next, pad1, pad2;   // r_next: request of entry0 + 1
};
struct ReqPos {
  int32_t first_pos, tiles;
};
struct StreamHeader {
  int32_t total_tiles, n_entries, n_waves, waves_used;
};
struct ReduceDesc {          // the segment cut by the boundary in front of work-group b
  int32_t n_parts;           // work-groups the segment spans (0: no segment is cut here)
  int32_t r, g, b0;          // segment and the first work-group it touches; boundary b0 + 1 owns its merge
};

constexpr int STREAM_MAX_WG = 4096;  // work-groups the pool workspace is sized for

// Shares of the tile stream.  Wave W of the `used` waves gets the tiles [start(W), start(W + 1)).
//   * Fewer tiles than waves: the empty ranges are all on the LEFT (wave W gets tile total - (used - W)), never
//     between two waves that hold tiles.  The attention kernel relies on this: a wave whose segment runs on past its
//     range waits for the first piece of its right-hand neighbour, and an empty wave never hands one over.
//   * Otherwise start(W) = floor(total * weight(0..W) / weight(all)): shares differ by at most one tile with equal
//     weights.  Work-groups on odd XCDs and the second wave on a SIMD (waves wpw/2.. of an 8-wave work-group) can be
//     given other weights (in 1/256 of the others'); weights are ignored below four tiles per wave, where a light
//     share could round to nothing.
// Weights are kept in 1/64 so that total (< 2^31) * cum (< 2^15 waves * 2^7 * 2^7) fits 64 bits.
struct StreamShares {
  int32_t total, used, wpw;
  long long w_even, w_odd, s_early, s_late, cum_all;

  ODMA_HD long long cum(int W) const {                     // weight of waves [0, W)
    const int half = wpw / 2;
    const long long s_wg = half * (s_early + s_late);       // slot weights of one whole work-group
    const int b = W / wpw, wv_in = W - b * wpw;
    const long long per8 = 4 * (w_even + w_odd);
    const int x = b & 7;                                    // work-group b runs on XCD b % 8
    const long long pre = (long long)(x + 1) / 2 * w_even + (long long)x / 2 * w_odd;   // work-groups before b in its round of 8
    const int early = wv_in < half ? wv_in : half, late = wv_in > half ? wv_in - half : 0;
    const long long in_wg = (long long)early * s_early + (long long)late * s_late;
    return ((long long)(b >> 3) * per8 + pre) * s_wg + ((x & 1) ? w_odd : w_even) * in_wg;
  }
  ODMA_HD int start(int W) const {
    if (W >= used) return total;
    if (total < used) return total - (used - W) > 0 ? total - (used - W) : 0;
    return (int)((long long)total * cum(W) / cum_all);
  }
};

// Waves used: all of them unless that would leave less than q_min tiles per wave; a whole number of work-groups.
ODMA_HD inline StreamShares stream_shares(int total, int n_waves, int wpw, int q_min, int odd_xcd_weight,
                                          int late_wave_weight) {
  StreamShares s;
  int used = n_waves;
  if ((long long)used * q_min > total) used = total / q_min > 1 ? total / q_min : 1;
  used = (used + wpw - 1) / wpw * wpw;
  if (used > n_waves) used = n_waves;
  const bool weighted = (long long)total >= 4ll * used;
  s.total = total;
  s.used = used;
  s.wpw = wpw;
  s.w_even = 64;
  s.w_odd = weighted ? odd_xcd_weight >> 2 : 64;
  s.s_early = 64;
  s.s_late = weighted ? late_wave_weight >> 2 : 64;
  s.cum_all = 1;
  s.cum_all = s.cum(used);
  return s;
}

// Byte offsets of the regions of a tile-stream workspace sized for max_requests requests, n_wg_cap attention
// work-groups and n_q_heads query heads (partial states keep 128 channels per head).
struct StreamLayout {
  size_t header, req_info, items, waves, red, arrive, part_ml, part_o, end;
};
ODMA_HD inline StreamLayout stream_layout(size_t off, int64_t max_requests, int64_t n_wg_cap, int64_t n_q_heads) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  StreamLayout w;
  w.header = off;   off += 256;
  w.req_info = off; off += up((size_t)max_requests * sizeof(ReqPos));
  w.items = off;    off += up((size_t)max_requests * sizeof(StreamEntry));
  w.waves = off;    off += up((size_t)n_wg_cap * 8 * sizeof(WaveDesc));
  w.red = off;      off += up((size_t)(n_wg_cap + 1) * sizeof(ReduceDesc));
  w.arrive = off;   off += up((size_t)(n_wg_cap + 1) * sizeof(int32_t));
  w.part_ml = off;  off += up((size_t)2 * n_wg_cap * n_q_heads * 2 * sizeof(float));
  w.part_o = off;   off += up((size_t)2 * n_wg_cap * n_q_heads * 128 * sizeof(float));
  w.end = off;
  return w;
}

}  // namespace odma_plan
