// Device side of libodma for gfx950 (MI355X): entry points that launch the kernels in
// decode_mfma.h (matrix-core decode attention over a balanced tile stream), decode_valu.h
// (fp32 vector-ALU decode attention over a chunked work list) and kv_rows.h (append,
// export, migration copy).
//
// Decode attention is a streaming scan of K and V with no reuse, so it is bounded by HBM
// bandwidth; both kernels keep the online-softmax state of a (request, KV head) range in
// registers, share each K/V byte among the query heads of its GQA group, and merge ranges
// of one request by log-sum-exp.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <mutex>
#include <string>

#include "odma_internal.h"
#include "kernels_common.h"
#include "decode_mfma.h"
#include "decode_valu.h"
#include "prefill_mfma.h"
#include "kv_rows.h"

namespace {

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
  if (layer < 0 || layer >= pool->cfg.n_layers || n < 0 || n > pool->cfg.max_requests || n > 65535 || !positions || !k_new || !v_new ||
      (!block_table && !offsets) || (block_table && bt_stride <= 0) || (n_new && !src_start) || max_new < 1 ||
      (!n_new && max_new != 1)) {
    odma::set_error("odma_append_kv: invalid argument");
    return ODMA_INVALID_ARG;
  }
  RowArgs a = row_args(pool, layer);
  const int groups = (max_new + BLK - 1) / BLK;
  dim3 grid(groups < APPEND_GRID_X ? groups : APPEND_GRID_X, n);
  hipStream_t s = (hipStream_t)stream;
  if (pool->elem_bytes == 1)
    hipLaunchKernelGGL(append_fp8_kernel, grid, dim3(256), 0, s, a, n, offsets, positions, 0, n_new, src_start,
                       block_table, bt_stride, (const unsigned char*)k_new, (const unsigned char*)v_new);
  else if (pool->elem_bytes == 2 && pool->cfg.head_dim == 128)
    hipLaunchKernelGGL(append_bf16_d128_kernel, grid, dim3(256), 0, s, a, n, offsets, positions, 0, n_new, src_start,
                       block_table, bt_stride, (const unsigned short*)k_new, (const unsigned short*)v_new);
  else if (pool->elem_bytes == 2)
    hipLaunchKernelGGL(append_kernel<unsigned short>, grid, dim3(256), 0, s, a, n, offsets, positions, 0, n_new, src_start,
                       block_table, bt_stride, (const unsigned short*)k_new, (const unsigned short*)v_new);
  else
    hipLaunchKernelGGL(append_kernel<float>, grid, dim3(256), 0, s, a, n, offsets, positions, 0, n_new, src_start,
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
  if (pool->elem_bytes == 1)
    hipLaunchKernelGGL(gather_fp8_kernel, grid, dim3(256), 0, s, a, offset, length, block_row, (unsigned char*)k_out,
                       (unsigned char*)v_out);
  else if (pool->elem_bytes == 2)
    hipLaunchKernelGGL(gather_kernel<unsigned short>, grid, dim3(256), 0, s, a, offset, length, block_row,
                       (unsigned short*)k_out, (unsigned short*)v_out);
  else
    hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(256), 0, s, a, offset, length, block_row, (float*)k_out,
                       (float*)v_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_gather_kv", e);
  return ODMA_OK;
}

int odma_prefill_attention(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, int64_t total_q,
                           const int64_t* q_start, const int32_t* n_q, const int64_t* offsets, const int32_t* lengths,
                           const int32_t* block_table, int32_t bt_stride, void* out, void* stream) {
  const char* where = "odma_prefill_attention";
  int rc = device_ready(pool, where);
  if (rc) return rc;
  const odma_pool_config_t& c = pool->cfg;
  if (pool->decode_kernel != ODMA_KERNEL_MFMA || c.head_dim != 128) {
    odma::set_error(std::string(where) + ": needs a bf16 or fp8 pool with head_dim 128 (the matrix-core path)");
    return ODMA_INVALID_ARG;
  }
  if (n == 0 || total_q == 0) return ODMA_OK;
  if (!c.workspace) {
    odma::set_error(std::string(where) + ": pool has no workspace");
    return ODMA_INVALID_ARG;
  }
  if (layer < 0 || layer >= c.n_layers || n < 0 || n > c.max_requests || total_q < 0 || !q || !q_start || !n_q ||
      !lengths || !out || (!block_table && !offsets) || (block_table && bt_stride <= 0)) {
    odma::set_error(std::string(where) + ": invalid argument");
    return ODMA_INVALID_ARG;
  }
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)c.workspace;
  const RowArgs ra = row_args(pool, layer);
  PrefillArgs a;
  a.k = ra.k;
  a.v = ra.v;
  a.q = (const unsigned short*)q;
  a.out = out;
  a.q_start = q_start;
  a.n_q = n_q;
  a.offsets = offsets;
  a.lengths = lengths;
  a.bt = block_table;
  a.bt_stride = bt_stride;
  a.hdr = (PrefillHeader*)(ws + pool->ws.prefill);
  a.item_start = (const int32_t*)(ws + pool->ws.prefill + 256);
  a.n = n;
  a.Hq = c.n_q_heads;
  a.Hkv = c.n_kv_heads;
  a.G = c.n_q_heads / c.n_kv_heads;
  a.total_q = total_q;
  a.head_stride = ra.head_stride;
  const bool fp8 = pool->elem_bytes == 1;
  a.scale_log2 = c.sm_scale * 1.4426950408889634f * (fp8 ? c.k_scale : 1.0f);
  a.out_scale = fp8 ? c.v_scale : 1.0f;
  a.out_bf16 = c.out_dtype == ODMA_BF16;
  // column tiles per wave: 2 (128-column items, two work-groups per CU whose LDS and matrix phases overlap)
  // measured faster than 4 (256-column items, one work-group per CU) on every prompt mix tried
  const int ct = pool->prefill_ct ? pool->prefill_ct : 2;
  hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(PREFILL_PLAN_THREADS), 0, s, n_q, lengths, q_start, total_q, n,
                     c.n_kv_heads, a.G, 64 * ct, a.hdr, (int32_t*)(ws + pool->ws.prefill + 256));
  const dim3 grid(pool->n_cu * (ct == 2 ? 2 : 1));
#ifdef ODMA_DEV_MINIMAL_VARIANTS
  odma::set_error(std::string(where) + ": not compiled into this development build");
  return ODMA_INVALID_ARG;
#else
  switch ((fp8 ? 4 : 0) + (ct == 2 ? 2 : 0) + (block_table ? 1 : 0)) {
    case 0: hipLaunchKernelGGL((prefill_kernel<false, 4, false>), grid, dim3(256), 0, s, a); break;
    case 1: hipLaunchKernelGGL((prefill_kernel<true, 4, false>), grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((prefill_kernel<false, 2, false>), grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL((prefill_kernel<true, 2, false>), grid, dim3(256), 0, s, a); break;
    case 4: hipLaunchKernelGGL((prefill_kernel<false, 4, true>), grid, dim3(256), 0, s, a); break;
    case 5: hipLaunchKernelGGL((prefill_kernel<true, 4, true>), grid, dim3(256), 0, s, a); break;
    case 6: hipLaunchKernelGGL((prefill_kernel<false, 2, true>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((prefill_kernel<true, 2, true>), grid, dim3(256), 0, s, a); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(where, e);
  return ODMA_OK;
#endif
}

int odma_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes == 0 || bytes % 16) {
    odma::set_error("odma_stream_read_probe: invalid argument");
    return ODMA_INVALID_ARG;
  }
  int dev = 0, n_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail("odma_stream_read_probe", e);
  hipLaunchKernelGGL(read_probe_kernel, dim3(n_cu > 0 ? n_cu : 256), dim3(256), 0, (hipStream_t)stream,
                     (const uint4v*)buf, bytes / 16, (unsigned*)sink);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_stream_read_probe", e);
  return ODMA_OK;
}

int odma_block_read_probe(const void* k_plane, const void* v_plane, const int32_t* table, int64_t n_steps, void* sink,
                          void* stream) {
  if (!k_plane || !v_plane || !table || !sink || n_steps <= 0) {
    odma::set_error("odma_block_read_probe: invalid argument");
    return ODMA_INVALID_ARG;
  }
  int dev = 0, n_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail("odma_block_read_probe", e);
  hipLaunchKernelGGL(block_probe_kernel, dim3(n_cu > 0 ? n_cu : 256), dim3(256), 0, (hipStream_t)stream,
                     (const char*)k_plane, (const char*)v_plane, table, n_steps, (unsigned*)sink);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("odma_block_read_probe", e);
  return ODMA_OK;
}

}  // extern "C"

namespace {

// Every instantiation of the tile-stream attention kernel, indexed [format][fused][paged][3 - nbuf][wpw == 4],
// and per instantiation the largest dynamic LDS size enabled so far (the default limit is 64 KiB).
using StreamKernel = void (*)(StreamArgs);
#ifdef ODMA_DEV_MINIMAL_VARIANTS
// development builds: only the default launch shape of the bf16 / head_dim 128 format is compiled; every other entry
// is null and its launch fails with an error
#define ODMA_SK_W(F, U, P, N) {nullptr, (F == STREAM_BF16_D128 && N == 2) ? decode_stream_kernel<P, 2, 4, U, STREAM_BF16_D128> : nullptr}
#else
#define ODMA_SK_W(F, U, P, N) {decode_stream_kernel<P, N, 8, U, F>, decode_stream_kernel<P, N, 4, U, F>}
#endif
#define ODMA_SK_N(F, U, P) {ODMA_SK_W(F, U, P, 3), ODMA_SK_W(F, U, P, 2)}
#define ODMA_SK_P(F, U) {ODMA_SK_N(F, U, false), ODMA_SK_N(F, U, true)}
#define ODMA_SK_U(F) {ODMA_SK_P(F, false), ODMA_SK_P(F, true)}
const StreamKernel stream_kernels[3][2][2][2][2] = {ODMA_SK_U(STREAM_BF16_D128), ODMA_SK_U(STREAM_FP8_D128),
                                                    ODMA_SK_U(STREAM_BF16_D64)};
std::atomic<unsigned> stream_kernel_lds[3][2][2][2][2];   // zero-initialised: nothing enabled beyond the default

hipError_t launch_stream_kernel(int fmt, bool fused, bool paged, int nbuf, int wpw, int n_wg, size_t lds_bytes,
                                hipStream_t s, const StreamArgs& a) {
  if (fmt < 0 || fmt > 2 || (nbuf != 2 && nbuf != 3) || (wpw != 4 && wpw != 8)) return hipErrorInvalidValue;
  const StreamKernel kernel = stream_kernels[fmt][fused][paged][3 - nbuf][wpw == 4];
  if (!kernel) return hipErrorInvalidDeviceFunction;
  std::atomic<unsigned>& allowed = stream_kernel_lds[fmt][fused][paged][3 - nbuf][wpw == 4];
  if (lds_bytes > 64 * 1024 && lds_bytes > allowed.load(std::memory_order_acquire)) {
    // racing callers may both set the attribute; the larger request wins in the end because each sets its own size
    // and then records the maximum
    const hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    unsigned seen = allowed.load(std::memory_order_relaxed);
    while (seen < lds_bytes && !allowed.compare_exchange_weak(seen, (unsigned)lds_bytes, std::memory_order_release)) {
    }
  }
  hipLaunchKernelGGL(kernel, dim3(n_wg), dim3(64 * wpw), lds_bytes, s, a);
  return hipSuccess;
}

// Static scratch of odma_decode_attention_static: plan records, arrival counters and partial states of one decode
// call, for callers that may not allocate.  Every GPU the library runs on holds its own copy of the array until the
// process ends.  In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device with that device current, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[ODMA_STATIC_SCRATCH_BYTES];

struct StaticScratch {
  char* ptr = nullptr;                     // device address of `scratch` on this device
  odma_pool::PlanStamp stamp;              // what the plan in it was made for (calls of every pool share it)
};
constexpr int STATIC_MAX_DEVICES = 64;
StaticScratch static_scratch[STATIC_MAX_DEVICES];
std::mutex static_scratch_mu;

int static_scratch_of_current_device(const char* where, StaticScratch** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(where, e);
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) {
    odma::set_error(std::string(where) + ": device ordinal out of range");
    return ODMA_INVALID_ARG;
  }
  std::lock_guard<std::mutex> lock(static_scratch_mu);
  StaticScratch& s = static_scratch[dev];
  if (!s.ptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(where, e);
    if (!p) {
      odma::set_error(std::string(where) + ": hipGetSymbolAddress returned no address");
      return ODMA_HIP_ERROR;
    }
    s.ptr = (char*)p;
  }
  *out = &s;
  return ODMA_OK;
}

// Where a decode call keeps its plan and partial states: the pool's workspace, or the library's static scratch.
struct DecodeScratch {
  char* base;
  odma::WorkspaceLayout layout;
  odma_pool::PlanStamp* stamp;             // what the plan in there was made for
  int n_wg_cap;                            // attention work-groups the regions are sized for
};

// Shared body of odma_decode_attention (k_new == nullptr), odma_decode_step and odma_decode_attention_static.
int decode_impl(const char* where, odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const void* k_new,
                const void* v_new, const int64_t* offsets, const int32_t* lengths, const int32_t* block_table,
                int32_t bt_stride, void* out, uint32_t flags, void* stream, const DecodeScratch* scratch = nullptr) {
  int rc = device_ready(pool, where);
  if (rc) return rc;
  if (n == 0) return ODMA_OK;
  const odma_pool_config_t& c = pool->cfg;
  if (!scratch && !c.workspace) {
    odma::set_error(std::string(where) + ": pool has no workspace");
    return ODMA_INVALID_ARG;
  }
  if (layer < 0 || layer >= c.n_layers || n < 0 || n > c.max_requests || !q || !lengths || !out ||
      (!block_table && !offsets) || (block_table && bt_stride <= 0)) {
    odma::set_error(std::string(where) + ": invalid argument");
    return ODMA_INVALID_ARG;
  }
  hipStream_t s = (hipStream_t)stream;
  char* ws = scratch ? scratch->base : (char*)c.workspace;
  const odma::WorkspaceLayout& wl = scratch ? scratch->layout : pool->ws;
  odma_pool::PlanStamp& stamp = scratch ? *scratch->stamp : pool->plan_stamp;
  const bool fp8 = pool->elem_bytes == 1;
  const bool d64 = pool->decode_kernel == ODMA_KERNEL_MFMA && c.head_dim == 64;
  const bool fused = k_new != nullptr && pool->decode_kernel == ODMA_KERNEL_MFMA;
  if (k_new && !fused) {
    // the vector-ALU path appends with the row kernel, then attends
    RowArgs wa = row_args(pool, layer);
    dim3 grid(1, n);
    if (fp8)
      hipLaunchKernelGGL(append_fp8_kernel, grid, dim3(256), 0, s, wa, n, offsets, lengths, -1,
                         (const int32_t*)nullptr, (const int64_t*)nullptr, block_table, bt_stride,
                         (const unsigned char*)k_new, (const unsigned char*)v_new);
    else if (pool->elem_bytes == 2)
      hipLaunchKernelGGL(append_kernel<unsigned short>, grid, dim3(256), 0, s, wa, n, offsets, lengths, -1,
                         (const int32_t*)nullptr, (const int64_t*)nullptr, block_table, bt_stride,
                         (const unsigned short*)k_new, (const unsigned short*)v_new);
    else
      hipLaunchKernelGGL(append_kernel<float>, grid, dim3(256), 0, s, wa, n, offsets, lengths, -1,
                         (const int32_t*)nullptr, (const int64_t*)nullptr, block_table, bt_stride, (const float*)k_new,
                         (const float*)v_new);
  }
  const RowArgs ra = row_args(pool, layer);
  const float scale_log2 = c.sm_scale * 1.4426950408889634f;
  const int G = c.n_q_heads / c.n_kv_heads;

  if (pool->decode_kernel == ODMA_KERNEL_MFMA) {
    // ---- tile-stream scheme: plan -> attention (one equal tile range per wave) -> reduce
    // Launch shape: one wave per SIMD (4 per CU, 4-wave work-groups) streams fastest, for both layouts.
    int wpw = pool->waves_per_wg ? pool->waves_per_wg : 4;
    const int wpc = pool->waves_per_cu ? pool->waves_per_cu : 4;
    // per-wave LDS queues: deep enough for the segments a wave of this launch shape typically finishes,
    // shallower (down to one entry) when a large GQA group makes the entries big
    int qs = 3, aq = wpw == 4 ? 6 : 3;
    while (qs > 1 && stream_lds_bytes(G, wpw, qs, aq) > 144 * 1024) --qs;
    if (stream_lds_bytes(G, wpw, qs, aq) > 160 * 1024) wpw = 4;
    int n_wg = pool->n_cu * wpc / wpw;
    if (n_wg > STREAM_MAX_WG) n_wg = STREAM_MAX_WG;
    if (n_wg < 1) n_wg = 1;
    if (scratch && n_wg > scratch->n_wg_cap) {
      odma::set_error(std::string(where) + ": the launch shape needs more work-groups than the static scratch holds");
      return ODMA_INVALID_ARG;
    }
    StreamArgs a;
    a.k = ra.k;
    a.v = ra.v;
    a.q = (const unsigned short*)q;
    a.out = out;
    a.k_new = k_new;
    a.v_new = v_new;
    a.bt = block_table;
    a.bt_stride = bt_stride;
    a.hdr = (const StreamHeader*)(ws + wl.header);
    a.entries = (const StreamEntry*)(ws + wl.items);
    a.waves = (const WaveDesc*)(ws + wl.waves);
    a.req_pos = (const ReqPos*)(ws + wl.req_info);
    a.red = (const ReduceDesc*)(ws + wl.red);
    a.arrive = (int32_t*)(ws + wl.arrive);
    a.fuse_reduce = pool->fuse_reduce && !(flags & ODMA_SKIP_REDUCE);
    a.part_ml = (float2*)(ws + wl.part_ml);
    a.part_o = (float*)(ws + wl.part_o);
    a.n = n;
    a.Hq = c.n_q_heads;
    a.Hkv = c.n_kv_heads;
    a.G = G;
    a.wpw = wpw;
    a.qs = qs;
    a.aq = aq;
    a.head_stride = ra.head_stride;
    // fp8 storage: stored values are value / k_scale and value / v_scale, and the kernel carries the
    // softmax weights times 256 through the matrix cores
    a.scale_log2 = fp8 ? scale_log2 * c.k_scale : scale_log2;
    a.out_scale = fp8 ? c.v_scale * (1.0f / 256.0f) : 1.0f;
    a.head_dim = c.head_dim;
    a.out_bf16 = c.out_dtype == ODMA_BF16;
    const int tile_tokens = (fp8 || d64) ? 2 * BLK : BLK;
    // A plan bakes in the slab bases and the launch shape, so ODMA_REUSE_PLAN is honoured only while the library
    // knows of nothing that changed them; otherwise the call plans again.
    const int q_min = pool->min_chunk ? (pool->min_chunk + tile_tokens - 1) / tile_tokens : 4;
    odma_pool::PlanStamp now;
    now.layout_gen = pool->layout_gen;
    now.owner = pool->serial;
    now.n = n;
    now.paged = block_table ? 1 : 0;
    now.n_wg = n_wg;
    now.wpw = wpw;
    now.q_min = q_min;
    now.tile_tokens = tile_tokens;
    now.odd_w = pool->odd_xcd_weight;
    now.late_w = wpw == 8 ? pool->late_wave_weight : 256;
    const odma_pool::PlanStamp& was = stamp;
    const bool reuse = (flags & ODMA_REUSE_PLAN) && was.layout_gen == now.layout_gen && was.owner == now.owner && was.n == now.n &&
                       was.paged == now.paged && was.n_wg == now.n_wg && was.wpw == now.wpw && was.q_min == now.q_min &&
                       was.tile_tokens == now.tile_tokens && was.odd_w == now.odd_w && was.late_w == now.late_w;
    if (!reuse) {
      hipLaunchKernelGGL(stream_plan_kernel, dim3(1), dim3(STREAM_PLAN_THREADS), 0, s, lengths,
                         block_table ? nullptr : offsets, n, c.n_kv_heads, tile_tokens, n_wg * wpw, wpw, q_min,
                         now.odd_w, now.late_w, (StreamHeader*)(ws + wl.header),
                         (StreamEntry*)(ws + wl.items), (WaveDesc*)(ws + wl.waves),
                         (ReqPos*)(ws + wl.req_info), (ReduceDesc*)(ws + wl.red),
                         (int32_t*)(ws + wl.arrive));
      stamp = now;
    }
    const size_t lds_bytes = stream_lds_bytes(G, wpw, qs, aq);
    const int nbuf = pool->pipeline_depth;
    const int fmt = d64 ? STREAM_BF16_D64 : fp8 ? STREAM_FP8_D128 : STREAM_BF16_D128;
    hipError_t e = launch_stream_kernel(fmt, fused, block_table != nullptr, nbuf, wpw, n_wg, lds_bytes, s, a);
    if (e != hipSuccess) return hip_fail(where, e);
    if (!pool->fuse_reduce && !(flags & ODMA_SKIP_REDUCE))
      hipLaunchKernelGGL(stream_reduce_kernel, dim3(n_wg * G), dim3(128), 0, s, a, n_wg);
  } else {
    // ---- chunked scheme: plan -> attention (one wave per (request, head, chunk)) -> reduce
    DecodeArgs a;
    a.k = ra.k;
    a.v = ra.v;
    a.q = q;
    a.out = out;
    a.offsets = offsets;
    a.lengths = lengths;
    a.bt = block_table;
    a.bt_stride = bt_stride;
    a.hdr = (const PlanHeader*)(ws + wl.header);
    a.items = (const Item*)(ws + wl.items);
    a.req = (const ReqInfo*)(ws + wl.req_info);
    a.part_ml = (float2*)(ws + wl.part_ml);
    a.part_o = (float*)(ws + wl.part_o);
    a.n = n;
    a.Hq = c.n_q_heads;
    a.Hkv = c.n_kv_heads;
    a.G = G;
    a.D = c.head_dim;
    a.head_stride = ra.head_stride;
    a.scale_log2 = scale_log2;
    a.out_bf16 = c.out_dtype == ODMA_BF16;
    const int waves = pool->n_cu * (pool->waves_per_cu ? pool->waves_per_cu : 8);
    if (!(flags & ODMA_REUSE_PLAN)) {
      const int target_pairs =
          (int)(((int64_t)waves * pool->items_per_wave_x16 / 16 + c.n_kv_heads - 1) / c.n_kv_heads);
      const int min_chunk = pool->min_chunk ? pool->min_chunk : 64;
      hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, lengths, n, target_pairs, min_chunk,
                         (int32_t)wl.max_pairs, (PlanHeader*)(ws + wl.header),
                         (ReqInfo*)(ws + wl.req_info), (Item*)(ws + wl.items));
    }
    dim3 grid(waves);
    if (pool->elem_bytes == 2) {
      if (block_table) hipLaunchKernelGGL((decode_valu_kernel<unsigned short, true>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((decode_valu_kernel<unsigned short, false>), grid, dim3(64), 0, s, a);
    } else {
      if (block_table) hipLaunchKernelGGL((decode_valu_kernel<float, true>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((decode_valu_kernel<float, false>), grid, dim3(64), 0, s, a);
    }
    if (!(flags & ODMA_SKIP_REDUCE))
      hipLaunchKernelGGL(reduce_kernel, dim3((n * c.n_q_heads + 3) / 4), dim3(256), 0, s, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(where, e);
  return ODMA_OK;
}

}  // namespace

extern "C" {

int odma_decode_attention(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const int64_t* offsets,
                          const int32_t* lengths, const int32_t* block_table, int32_t bt_stride, void* out,
                          uint32_t flags, void* stream) {
  return decode_impl("odma_decode_attention", pool, layer, n, q, nullptr, nullptr, offsets, lengths, block_table,
                     bt_stride, out, flags, stream);
}

int odma_decode_step(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const void* k_new, const void* v_new,
                     const int64_t* offsets, const int32_t* lengths, const int32_t* block_table, int32_t bt_stride,
                     void* out, uint32_t flags, void* stream) {
  if (!k_new || !v_new) {
    odma::set_error("odma_decode_step: k_new and v_new are required");
    return ODMA_INVALID_ARG;
  }
  return decode_impl("odma_decode_step", pool, layer, n, q, k_new, v_new, offsets, lengths, block_table, bt_stride,
                     out, flags, stream);
}

int odma_decode_attention_static(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const int64_t* offsets,
                                 const int32_t* lengths, const int32_t* block_table, int32_t bt_stride, void* out,
                                 uint32_t flags, void* stream) {
  const char* where = "odma_decode_attention_static";
  int rc = device_ready(pool, where);
  if (rc) return rc;
  if (pool->decode_kernel != ODMA_KERNEL_MFMA) {
    odma::set_error(std::string(where) + ": serves the matrix-core kernel only (bf16 or fp8 pools, head_dim 128 or 64)");
    return ODMA_INVALID_ARG;
  }
  if (flags & ~(uint32_t)ODMA_REUSE_PLAN) {
    odma::set_error(std::string(where) + ": the only flag accepted is ODMA_REUSE_PLAN");
    return ODMA_INVALID_ARG;
  }
  if (n < 0 || n > ODMA_STATIC_MAX_REQUESTS) {
    odma::set_error(std::string(where) + ": n exceeds ODMA_STATIC_MAX_REQUESTS");
    return ODMA_INVALID_ARG;
  }
  const odma_plan::StreamLayout sl =
      odma_plan::stream_layout(0, ODMA_STATIC_MAX_REQUESTS, ODMA_STATIC_MAX_WORKGROUPS, pool->cfg.n_q_heads);
  if (sl.end > ODMA_STATIC_SCRATCH_BYTES) {
    odma::set_error(std::string(where) + ": too many query heads for the static scratch (ODMA_STATIC_SCRATCH_BYTES)");
    return ODMA_INVALID_ARG;
  }
  StaticScratch* dev = nullptr;
  rc = static_scratch_of_current_device(where, &dev);
  if (rc) return rc;
  DecodeScratch sc;
  sc.base = dev->ptr;
  sc.layout.header = sl.header;
  sc.layout.req_info = sl.req_info;
  sc.layout.items = sl.items;
  sc.layout.waves = sl.waves;
  sc.layout.red = sl.red;
  sc.layout.arrive = sl.arrive;
  sc.layout.part_ml = sl.part_ml;
  sc.layout.part_o = sl.part_o;
  sc.layout.total = sl.end;
  sc.stamp = &dev->stamp;
  sc.n_wg_cap = ODMA_STATIC_MAX_WORKGROUPS;
  return decode_impl(where, pool, layer, n, q, nullptr, nullptr, offsets, lengths, block_table, bt_stride, out, flags,
                     stream, &sc);
}

#ifdef ODMA_DEV_TIMELINE
int odma_dev_timeline(long long* host_dst, size_t n_values) {
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(odma_dev_timeline_buf), n_values * sizeof(long long));
  return e == hipSuccess ? ODMA_OK : hip_fail("odma_dev_timeline", e);
}
#endif

}  // extern "C"

namespace {
// Device half of odma_migrate / odma_migrate_batch (the bookkeeping is in the host half): one launch copies, for
// every layer, K and V, the byte runs of up to MIGRATE_BATCH_MAX requests.  Installed below as odma::migrate_copy.
int launch_migrate_copy(odma_pool* pool, int32_t n, const int64_t* src_byte, const int64_t* dst_byte, const int64_t* n_bytes,
                        void* stream) {
  const int64_t block_bytes = (int64_t)BLK * pool->cfg.head_dim * pool->elem_bytes;
  const int64_t plane_stride = pool->pool_blocks * block_bytes;
  const int planes = pool->cfg.n_layers * pool->cfg.n_kv_heads;
  const int64_t per_block_bytes = 256 * 16 * 8;
  for (int32_t i0 = 0; i0 < n; i0 += MIGRATE_BATCH_MAX) {
    MigrateBatch mb;
    mb.n = n - i0 < MIGRATE_BATCH_MAX ? n - i0 : MIGRATE_BATCH_MAX;
    int64_t longest = 0;
    for (int32_t i = 0; i < mb.n; ++i) {
      mb.src_byte[i] = src_byte[i0 + i];
      mb.dst_byte[i] = dst_byte[i0 + i];
      mb.n_bytes[i] = n_bytes[i0 + i];
      longest = n_bytes[i0 + i] > longest ? n_bytes[i0 + i] : longest;
    }
    int gx = (int)((longest + per_block_bytes - 1) / per_block_bytes);
    gx = gx < 1 ? 1 : (gx > 1024 ? 1024 : gx);
    if (mb.n == 1)
      hipLaunchKernelGGL(migrate_copy_kernel, dim3(gx, planes * 2), dim3(256), 0, (hipStream_t)stream, (char*)pool->cfg.k_pool,
                         (char*)pool->cfg.v_pool, plane_stride, mb.src_byte[0], mb.dst_byte[0], mb.n_bytes[0]);
    else
      hipLaunchKernelGGL(migrate_batch_kernel, dim3(gx, planes * 2, mb.n), dim3(256), 0, (hipStream_t)stream,
                         (char*)pool->cfg.k_pool, (char*)pool->cfg.v_pool, plane_stride, mb);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("migration copy", e);
  return ODMA_OK;
}
const bool migrate_copy_installed = (odma::migrate_copy = &launch_migrate_copy, true);
}  // namespace

extern "C" {
}  // extern "C"
