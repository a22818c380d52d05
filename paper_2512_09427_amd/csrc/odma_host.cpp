// Host side of libodma: the ODMA allocator and its bookkeeping.
//
// Follows Section III of the paper: uncertainty-inflated length estimates routed to
// bucket slabs or the Large Bucket (III-B, III-D), contiguous reservation from
// per-arena free lists (III-A, III-E), overflow detection and allocate-and-copy
// migration bookkeeping (III-D, IV-C), quantile recalibration of the boundaries from
// a sliding-window histogram (III-C, Eq. 2), and the utilization totals of Section V.
// Everything here is integer arithmetic except odma_inflate (IEEE double, compiled
// without FMA contraction), so results are reproducible bit for bit.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "odma_internal.h"

namespace odma {

static thread_local std::string g_error;

void set_error(const std::string& msg) { g_error = msg; }

void Arena::init(int64_t b, int64_t s) {
  base = b;
  size = s;
  free_list.clear();
  if (s > 0) free_list.push_back({b, s});
}

int64_t Arena::reserve(int64_t cap) {
  for (size_t i = 0; i < free_list.size(); ++i) {
    if (free_list[i].size >= cap) {
      int64_t start = free_list[i].start;
      if (free_list[i].size == cap) {
        free_list.erase(free_list.begin() + i);
      } else {
        free_list[i].start += cap;
        free_list[i].size -= cap;
      }
      return start;
    }
  }
  return -1;
}

void Arena::release(int64_t off, int64_t cap) {
  auto it = std::lower_bound(free_list.begin(), free_list.end(), off,
                             [](const Extent& e, int64_t o) { return e.start < o; });
  size_t i = it - free_list.begin();
  free_list.insert(it, {off, cap});
  if (i + 1 < free_list.size() && free_list[i].start + free_list[i].size == free_list[i + 1].start) {
    free_list[i].size += free_list[i + 1].size;
    free_list.erase(free_list.begin() + i + 1);
  }
  if (i > 0 && free_list[i - 1].start + free_list[i - 1].size == free_list[i].start) {
    free_list[i - 1].size += free_list[i].size;
    free_list.erase(free_list.begin() + i);
  }
}

void Calibrator::push(int32_t realized_len) {
  const int32_t L = std::min(std::max(realized_len, 1), large_cap);
  const size_t W = ring.size();
  if (count == W) {
    const int32_t old = ring[head];
    hist[(old - 1) / align]--;
    ring[head] = L;
    head = (head + 1) % W;
  } else {
    ring[(head + count) % W] = L;
    count++;
  }
  hist[(L - 1) / align]++;
}

bool Calibrator::compute(int32_t* out, int32_t B) const {
  const int64_t cnt = (int64_t)count;
  if (cnt == 0) return false;
  std::vector<int64_t> b(B);
  for (int32_t i = 0; i < B; ++i) {
    int64_t k = ((int64_t)qnum[i] * cnt + qden[i] - 1) / qden[i];     // ceil(p_i * n), p_i rational
    if (k < 1) k = 1;
    int64_t cum = 0;
    size_t j = 0;
    for (; j < hist.size(); ++j) {
      cum += hist[j];
      if (cum >= k) break;
    }
    if (j >= hist.size()) j = hist.size() - 1;
    b[i] = (int64_t)(j + 1) * align;
  }
  for (int32_t i = 1; i < B; ++i) b[i] = std::max(b[i], b[i - 1] + align);
  b[B - 1] = std::min<int64_t>(b[B - 1], large_cap);
  for (int32_t i = B - 2; i >= 0; --i) b[i] = std::min(b[i], b[i + 1] - align);
  for (int32_t i = 0; i < B; ++i) out[i] = (int32_t)b[i];
  return true;
}

int64_t Arena::free_tokens() const {
  int64_t s = 0;
  for (const auto& e : free_list) s += e.size;
  return s;
}

static bool check_boundaries(const int32_t* b, int32_t n, int32_t align, int32_t large_cap) {
  if (!b || n <= 0) return false;
  int64_t prev = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (b[i] <= prev || b[i] % align != 0 || b[i] > large_cap) return false;
    prev = b[i];
  }
  return true;
}

bool validate_config(const odma_pool_config_t& c, std::string* why) {
  auto fail = [&](const char* m) {
    if (why) *why = m;
    return false;
  };
  if (c.n_layers <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0) return fail("layer/head counts must be positive");
  if (c.n_q_heads % c.n_kv_heads) return fail("n_q_heads must be a multiple of n_kv_heads");
  if (c.n_q_heads / c.n_kv_heads > 16) return fail("at most 16 query heads per KV head");
  if (c.head_dim <= 0 || c.head_dim % 32 || c.head_dim > 256) return fail("head_dim must be a multiple of 32, <= 256");
  if (c.kv_dtype != ODMA_F32 && c.kv_dtype != ODMA_BF16 && c.kv_dtype != ODMA_FP8) return fail("kv_dtype");
  if (c.kv_dtype == ODMA_FP8 && (c.head_dim != 128 || c.decode_kernel == ODMA_KERNEL_VALU))
    return fail("fp8 storage is served by the matrix-core kernel only: head_dim 128");
  if (!(c.k_scale >= 0.0f) || !(c.v_scale >= 0.0f)) return fail("k_scale and v_scale must be >= 0");
  if (c.out_dtype != ODMA_F32 && c.out_dtype != ODMA_BF16) return fail("out_dtype");
  if (c.align_tokens <= 0 || c.align_tokens % ODMA_BLOCK_TOKENS) return fail("align_tokens must be a multiple of 16");
  if (c.large_cap <= 0 || c.large_cap % c.align_tokens) return fail("large_cap must be a positive multiple of align_tokens");
  if (c.main_tokens < 0 || c.main_tokens % c.align_tokens) return fail("main_tokens must be a multiple of align_tokens");
  if (c.safety_tokens < 0 || c.safety_tokens % c.align_tokens) return fail("safety_tokens must be a multiple of align_tokens");
  if (c.main_tokens + c.safety_tokens <= 0) return fail("empty pool");
  if ((c.main_tokens + c.safety_tokens) / ODMA_BLOCK_TOKENS > INT32_MAX) return fail("pool too large for 32-bit block ids");
  if (c.max_requests <= 0) return fail("max_requests must be positive");
  if (c.n_buckets <= 0 || c.n_buckets > 64) return fail("n_buckets must be in 1..64");
  if (!check_boundaries(c.boundaries, c.n_buckets, c.align_tokens, c.large_cap))
    return fail("boundaries must be increasing multiples of align_tokens, <= large_cap");
  if ((c.quantile_num == nullptr) != (c.quantile_den == nullptr)) return fail("quantile_num and quantile_den go together");
  if (c.quantile_num) {
    for (int i = 0; i < c.n_buckets; ++i)
      if (c.quantile_den[i] <= 0 || c.quantile_num[i] <= 0 || c.quantile_num[i] > c.quantile_den[i])
        return fail("quantile levels must satisfy 0 < num/den <= 1");
  }
  if (c.window <= 0) return fail("window must be positive");
  if (!(c.gamma >= 0.0) || !(c.tau >= 0.0)) return fail("gamma and tau must be >= 0");
  if (c.decode_kernel < ODMA_KERNEL_AUTO || c.decode_kernel > ODMA_KERNEL_MFMA) return fail("decode_kernel");
  if (c.max_splits < 0) return fail("max_splits");
  if (c.decode_kernel == ODMA_KERNEL_MFMA &&
      !((c.kv_dtype == ODMA_BF16 && (c.head_dim == 128 || c.head_dim == 64)) || (c.kv_dtype == ODMA_FP8 && c.head_dim == 128)))
    return fail("the MFMA kernel needs bf16 storage with head_dim 128 or 64, or fp8 storage with head_dim 128");
  return true;
}

// Device workspace carve-up.  The chunked scheme (VALU kernel) and the tile-stream scheme (MFMA kernel) never run
// on the same pool, so each pool gets only the regions of its own.
WorkspaceLayout workspace_layout(const odma_pool_config_t& c) {
  using namespace odma_plan;
  WorkspaceLayout w;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off = 0;
  if (resolve_decode_kernel(c) == ODMA_KERNEL_MFMA) {
    const StreamLayout s = stream_layout(0, c.max_requests, STREAM_MAX_WG, c.n_q_heads);
    w.max_pairs = 0;
    w.header = s.header;
    w.req_info = s.req_info;
    w.items = s.items;
    w.waves = s.waves;
    w.red = s.red;
    w.arrive = s.arrive;
    w.part_ml = s.part_ml;
    w.part_o = s.part_o;
    off = s.end;
    // prefill attention: queue header and the exclusive prefix of work items per request
    w.prefill = off;  off += 256 + up((size_t)(c.max_requests + 1) * sizeof(int32_t));
  } else {
    w.header = off;
    off += 256;
    int64_t max_splits = c.max_splits > 0 ? c.max_splits : 8192;
    w.max_pairs = (int64_t)c.max_requests + max_splits;
    w.req_info = off; off += up((size_t)c.max_requests * sizeof(ReqInfo));
    w.items = off;    off += up((size_t)w.max_pairs * sizeof(Item));
    w.waves = off;
    w.part_ml = off;  off += up((size_t)w.max_pairs * c.n_q_heads * 2 * sizeof(float));
    w.part_o = off;   off += up((size_t)w.max_pairs * c.n_q_heads * c.head_dim * sizeof(float));
  }
  w.total = off;
  return w;
}

int resolve_decode_kernel(const odma_pool_config_t& c) {
  if (c.decode_kernel != ODMA_KERNEL_AUTO) return c.decode_kernel;
  const bool mfma = (c.kv_dtype == ODMA_BF16 && (c.head_dim == 128 || c.head_dim == 64)) || (c.kv_dtype == ODMA_FP8 && c.head_dim == 128);
  return mfma ? ODMA_KERNEL_MFMA : ODMA_KERNEL_VALU;
}

}  // namespace odma

using namespace odma;

// ---------------------------------------------------------------------------------
// background recalibration
// ---------------------------------------------------------------------------------
static void recalibrator_main(odma_pool* pool) {
  Recalibrator& rc = *pool->recal;
  const int32_t B = (int32_t)pool->boundaries.size();
  std::vector<int32_t> batch, b(B);
  int64_t folded = 0;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(rc.mu);
      rc.wake.wait(lk, [&] { return rc.stop || !rc.inbox.empty(); });
      if (rc.inbox.empty() && rc.stop) return;
      batch.swap(rc.inbox);
    }
    for (int32_t L : batch) {
      pool->calib.push(L);
      ++folded;
      if (folded % rc.refresh == 0 && pool->calib.compute(b.data(), B)) {
        // publish: odd sequence number while the set is being written
        const uint32_t s0 = rc.seq.load(std::memory_order_relaxed);
        rc.seq.store(s0 + 1, std::memory_order_relaxed);
        std::atomic_thread_fence(std::memory_order_release);
        for (int32_t i = 0; i < B; ++i) rc.pub_b[i].store(b[i], std::memory_order_relaxed);
        rc.pub_epoch.store(folded / rc.refresh, std::memory_order_relaxed);
        rc.seq.store(s0 + 2, std::memory_order_release);
      }
    }
    batch.clear();
    rc.folded.store(folded, std::memory_order_release);
    {
      std::lock_guard<std::mutex> lk(rc.mu);
      if (rc.inbox.empty()) rc.idle.notify_all();
    }
  }
}

// Takes the newest published boundaries, if any are newer than the ones in use.  Lock-free:
// a reader never blocks the worker, and retries only while a publication is in progress.
static void adopt_published(odma_pool* pool) {
  Recalibrator& rc = *pool->recal;
  const int32_t B = (int32_t)pool->boundaries.size();
  int32_t b[64];
  int64_t epoch;
  for (;;) {
    const uint32_t s0 = rc.seq.load(std::memory_order_acquire);
    if (s0 & 1) continue;
    epoch = rc.pub_epoch.load(std::memory_order_relaxed);
    for (int32_t i = 0; i < B; ++i) b[i] = rc.pub_b[i].load(std::memory_order_relaxed);
    std::atomic_thread_fence(std::memory_order_acquire);
    if (rc.seq.load(std::memory_order_relaxed) == s0) break;
  }
  if (epoch > pool->boundary_epoch) {
    for (int32_t i = 0; i < B; ++i) pool->boundaries[i] = b[i];
    pool->stats.recalibrations += epoch - pool->boundary_epoch;
    pool->boundary_epoch = epoch;
  }
}

extern "C" {

const char* odma_last_error(void) { return g_error.c_str(); }
const char* odma_version(void) { return "libodma 0.1 (gfx950)"; }

size_t odma_workspace_bytes(const odma_pool_config_t* cfg) {
  if (!cfg) return 0;
  // boundaries are not needed to size the workspace: validate the geometry only
  odma_pool_config_t c = *cfg;
  int32_t one = c.align_tokens > 0 ? c.align_tokens : 16;
  if (!c.boundaries) {
    c.boundaries = &one;
    c.n_buckets = 1;
    c.quantile_num = c.quantile_den = nullptr;
  }
  std::string why;
  if (!validate_config(c, &why)) {
    set_error("odma_workspace_bytes: " + why);
    return 0;
  }
  return workspace_layout(c).total;
}

int odma_pool_create(const odma_pool_config_t* cfg, odma_pool_t** out) {
  if (!cfg || !out) {
    set_error("odma_pool_create: null argument");
    return ODMA_INVALID_ARG;
  }
  *out = nullptr;
  std::string why;
  if (!validate_config(*cfg, &why)) {
    set_error("odma_pool_create: " + why);
    return ODMA_INVALID_ARG;
  }
  odma_pool* p = new (std::nothrow) odma_pool();
  if (!p) {
    set_error("odma_pool_create: out of host memory");
    return ODMA_NOMEM;
  }
  static std::atomic<uint64_t> next_serial{1};
  p->serial = next_serial.fetch_add(1, std::memory_order_relaxed);
  p->cfg = *cfg;
  p->boundaries.assign(cfg->boundaries, cfg->boundaries + cfg->n_buckets);
  Calibrator& cal = p->calib;
  if (cfg->quantile_num) {
    cal.qnum.assign(cfg->quantile_num, cfg->quantile_num + cfg->n_buckets);
    cal.qden.assign(cfg->quantile_den, cfg->quantile_den + cfg->n_buckets);
  } else if (cfg->n_buckets == 4) {
    cal.qnum = {1, 4, 19, 99};
    cal.qden = {2, 5, 20, 100};
  } else if (cfg->n_buckets == 3) {
    cal.qnum = {1, 9, 99};
    cal.qden = {2, 10, 100};
  }
  cal.align = cfg->align_tokens;
  cal.large_cap = cfg->large_cap;
  p->cfg.boundaries = nullptr;
  p->cfg.quantile_num = p->cfg.quantile_den = nullptr;
  if (p->cfg.sm_scale == 0.0f) p->cfg.sm_scale = 1.0f / std::sqrt((float)cfg->head_dim);
  p->arenas[0].init(0, cfg->main_tokens);
  p->arenas[1].init(cfg->main_tokens, cfg->safety_tokens);
  p->req.assign(cfg->max_requests, Request());
  cal.ring.assign(cfg->window, 0);
  cal.hist.assign(cfg->large_cap / cfg->align_tokens, 0);
  p->ws = workspace_layout(*cfg);
  p->decode_kernel = resolve_decode_kernel(*cfg);
  p->pool_blocks = (cfg->main_tokens + cfg->safety_tokens) / ODMA_BLOCK_TOKENS;
  p->elem_bytes = cfg->kv_dtype == ODMA_FP8 ? 1 : cfg->kv_dtype == ODMA_BF16 ? 2 : 4;
  if (p->cfg.k_scale == 0.0f) p->cfg.k_scale = 1.0f;
  if (p->cfg.v_scale == 0.0f) p->cfg.v_scale = 1.0f;
  if (cfg->workspace && cfg->workspace_bytes < p->ws.total) {
    set_error("odma_pool_create: workspace smaller than odma_workspace_bytes()");
    delete p;
    return ODMA_INVALID_ARG;
  }
  if (cfg->workspace && ((uintptr_t)cfg->workspace & 255)) {
    set_error("odma_pool_create: workspace must be 256-byte aligned");
    delete p;
    return ODMA_INVALID_ARG;
  }
  if ((cfg->k_pool && ((uintptr_t)cfg->k_pool & 255)) || (cfg->v_pool && ((uintptr_t)cfg->v_pool & 255))) {
    set_error("odma_pool_create: k_pool and v_pool must be 256-byte aligned");
    delete p;
    return ODMA_INVALID_ARG;
  }
  p->stats.main_free = cfg->main_tokens;
  p->stats.safety_free = cfg->safety_tokens;
  *out = p;
  return ODMA_OK;
}

int odma_pool_destroy(odma_pool_t* pool) {
  if (pool && pool->recal) odma_recalibrator_stop(pool);
  delete pool;
  return ODMA_OK;
}

int64_t odma_inflate(const odma_pool_t* pool, int32_t pred_len, float u) {
  if (!pool) return -1;
  double grown = (double)pred_len * (1.0 + pool->cfg.gamma * (double)u);
  return (int64_t)std::ceil(grown);
}

int odma_assign(odma_pool_t* pool, int32_t n, const int32_t* req_id, const int32_t* pred_len,
                const float* uncertainty, const int32_t* prompt_len,
                const int32_t* boundaries, int32_t n_boundaries,
                int32_t* bucket, int64_t* offset, int32_t* cap, int32_t* status) {
  if (!pool || n < 0 || (n > 0 && (!req_id || !pred_len || !bucket || !offset || !cap || !status))) {
    set_error("odma_assign: null argument");
    return ODMA_INVALID_ARG;
  }
  if (pool->recal) adopt_published(pool);
  const int32_t* b = pool->boundaries.data();
  int32_t nb = (int32_t)pool->boundaries.size();
  if (boundaries) {
    if (!check_boundaries(boundaries, n_boundaries, pool->cfg.align_tokens, pool->cfg.large_cap)) {
      for (int32_t i = 0; i < n; ++i) {
        bucket[i] = -1; offset[i] = -1; cap[i] = 0; status[i] = ODMA_INVALID_ARG;
      }
      set_error("odma_assign: boundaries must be increasing multiples of align_tokens, <= large_cap");
      return ODMA_INVALID_ARG;
    }
    b = boundaries;
    nb = n_boundaries;
  }
  int first_err = ODMA_OK;
  const int32_t large_cap = pool->cfg.large_cap;
  for (int32_t i = 0; i < n; ++i) {
    int32_t rid = req_id[i];
    float u = uncertainty ? uncertainty[i] : 0.0f;
    int64_t prompt = prompt_len ? prompt_len[i] : 0;
    int64_t pred = pred_len[i];
    int st = ODMA_OK;
    int32_t bk = -1, cp = 0;
    int64_t off = -1;
    if (rid < 0 || rid >= pool->cfg.max_requests || pred < 0 || prompt < 0 || !(u >= 0.0f && u <= 1.0f)) {
      st = ODMA_INVALID_ARG;
    } else if (pool->req[rid].arena >= 0) {
      st = ODMA_UNKNOWN_REQ;
    } else {
      int64_t need = prompt + (uncertainty ? odma_inflate(pool, (int32_t)pred, u) : pred);
      if (need < 1) need = 1;
      if (need > large_cap) {
        st = ODMA_OVERFLOW;
      } else {
        int arena;
        if ((double)u > pool->cfg.tau || need > b[nb - 1]) {
          bk = nb; cp = large_cap; arena = ODMA_ARENA_SAFETY;
        } else {
          int32_t j = 0;
          while (b[j] < need) ++j;
          bk = j; cp = b[j]; arena = ODMA_ARENA_MAIN;
        }
        int64_t got = pool->arenas[arena].reserve(cp);
        if (got < 0) {
          st = ODMA_NOMEM; bk = -1; cp = 0;
          pool->stats.nomem++;
        } else {
          off = got;
          Request& r = pool->req[rid];
          r.arena = arena; r.off = off; r.cap = cp; r.len = 0; r.left_behind = 0;
          pool->layout_gen++;
          pool->stats.live_requests++;
          pool->stats.live_reserved += cp;
        }
      }
    }
    bucket[i] = bk; offset[i] = off; cap[i] = cp; status[i] = st;
    if (st != ODMA_OK && first_err == ODMA_OK) first_err = st;
  }
  if (first_err != ODMA_OK) set_error("odma_assign: at least one request failed; see status[]");
  return first_err;
}

int odma_release(odma_pool_t* pool, int32_t n, const int32_t* req_id, int32_t* status) {
  if (!pool || n < 0 || (n > 0 && !req_id)) {
    set_error("odma_release: null argument");
    return ODMA_INVALID_ARG;
  }
  int first_err = ODMA_OK;
  for (int32_t i = 0; i < n; ++i) {
    int32_t rid = req_id[i];
    int st = ODMA_OK;
    if (rid < 0 || rid >= pool->cfg.max_requests || pool->req[rid].arena < 0) {
      st = ODMA_UNKNOWN_REQ;
    } else {
      Request& r = pool->req[rid];
      pool->layout_gen++;
      pool->arenas[r.arena].release(r.off, r.cap);
      if (r.held_arena >= 0) pool->arenas[r.held_arena].release(r.held_off, r.held_cap);
      pool->stats.live_requests--;
      pool->stats.live_tokens -= r.len;
      pool->stats.live_reserved -= r.cap;
      pool->stats.done_requests++;
      pool->stats.done_actual += r.len;
      pool->stats.done_reserved += r.cap;
      pool->stats.done_reserved_both += r.cap + r.left_behind;
      r = Request();
    }
    if (status) status[i] = st;
    if (st != ODMA_OK && first_err == ODMA_OK) first_err = st;
  }
  if (first_err != ODMA_OK) set_error("odma_release: unknown request id");
  return first_err;
}

int odma_advance(odma_pool_t* pool, int32_t n, const int32_t* req_id, const int32_t* n_new,
                 int32_t* overflow, int32_t* status) {
  if (!pool || n < 0 || (n > 0 && (!req_id || !overflow))) {
    set_error("odma_advance: null argument");
    return ODMA_INVALID_ARG;
  }
  int first_err = ODMA_OK;
  for (int32_t i = 0; i < n; ++i) {
    int32_t rid = req_id[i];
    int64_t k = n_new ? n_new[i] : 1;
    int st = ODMA_OK;
    overflow[i] = 0;
    if (rid < 0 || rid >= pool->cfg.max_requests || pool->req[rid].arena < 0) {
      st = ODMA_UNKNOWN_REQ;
    } else if (k < 0) {
      st = ODMA_INVALID_ARG;
    } else {
      Request& r = pool->req[rid];
      if ((int64_t)r.len + k > r.cap) {
        overflow[i] = 1;
      } else {
        r.len += (int32_t)k;
        pool->stats.live_tokens += k;
      }
    }
    if (status) status[i] = st;
    if (st != ODMA_OK && first_err == ODMA_OK) first_err = st;
  }
  if (first_err != ODMA_OK) set_error("odma_advance: at least one request failed; see status[]");
  return first_err;
}

int odma_recalibrate(odma_pool_t* pool, int32_t n, const int32_t* realized_len, int32_t* boundaries_out) {
  if (!pool || n < 0 || (n > 0 && !realized_len) || !boundaries_out) {
    set_error("odma_recalibrate: null argument");
    return ODMA_INVALID_ARG;
  }
  const int32_t B = (int32_t)pool->boundaries.size();
  if ((int32_t)pool->calib.qnum.size() != B) {
    set_error("odma_recalibrate: no quantile levels configured for this number of buckets");
    return ODMA_INVALID_ARG;
  }
  if (pool->recal) {
    set_error("odma_recalibrate: the background recalibrator owns the window; report completions to it");
    return ODMA_INVALID_ARG;
  }
  for (int32_t i = 0; i < n; ++i) pool->calib.push(realized_len[i]);
  if (pool->calib.compute(pool->boundaries.data(), B)) pool->stats.recalibrations++;
  std::memcpy(boundaries_out, pool->boundaries.data(), sizeof(int32_t) * B);
  return ODMA_OK;
}

int odma_recalibrator_start(odma_pool_t* pool, int32_t refresh_every) {
  if (!pool || refresh_every < 1) {
    set_error("odma_recalibrator_start: invalid argument");
    return ODMA_INVALID_ARG;
  }
  if (pool->recal) {
    set_error("odma_recalibrator_start: already running");
    return ODMA_INVALID_ARG;
  }
  if (pool->calib.qnum.size() != pool->boundaries.size()) {
    set_error("odma_recalibrator_start: no quantile levels configured for this number of buckets");
    return ODMA_INVALID_ARG;
  }
  pool->recal.reset(new (std::nothrow) Recalibrator());
  if (!pool->recal) {
    set_error("odma_recalibrator_start: out of host memory");
    return ODMA_NOMEM;
  }
  Recalibrator& rc = *pool->recal;
  rc.refresh = refresh_every;
  for (size_t i = 0; i < pool->boundaries.size(); ++i) rc.pub_b[i].store(pool->boundaries[i]);
  rc.pub_epoch.store(0);
  pool->boundary_epoch = 0;
  rc.worker = std::thread(recalibrator_main, pool);
  return ODMA_OK;
}

int odma_report_completions(odma_pool_t* pool, int32_t n, const int32_t* realized_len) {
  if (!pool || n < 0 || (n > 0 && !realized_len)) {
    set_error("odma_report_completions: invalid argument");
    return ODMA_INVALID_ARG;
  }
  if (!pool->recal) {
    set_error("odma_report_completions: no recalibrator is running (odma_recalibrator_start)");
    return ODMA_INVALID_ARG;
  }
  Recalibrator& rc = *pool->recal;
  {
    std::lock_guard<std::mutex> lk(rc.mu);
    rc.inbox.insert(rc.inbox.end(), realized_len, realized_len + n);
    rc.reported += n;
  }
  rc.wake.notify_one();
  return ODMA_OK;
}

int odma_recalibrator_drain(odma_pool_t* pool, int64_t* epoch) {
  if (!pool || !pool->recal) {
    set_error("odma_recalibrator_drain: no recalibrator is running");
    return ODMA_INVALID_ARG;
  }
  Recalibrator& rc = *pool->recal;
  {
    std::unique_lock<std::mutex> lk(rc.mu);
    rc.idle.wait(lk, [&] { return rc.inbox.empty() && rc.folded.load(std::memory_order_acquire) == rc.reported; });
  }
  if (epoch) *epoch = rc.pub_epoch.load(std::memory_order_acquire);
  return ODMA_OK;
}

int odma_recalibrator_stop(odma_pool_t* pool) {
  if (!pool || !pool->recal) {
    set_error("odma_recalibrator_stop: no recalibrator is running");
    return ODMA_INVALID_ARG;
  }
  Recalibrator& rc = *pool->recal;
  {
    std::lock_guard<std::mutex> lk(rc.mu);
    rc.stop = true;
  }
  rc.wake.notify_one();
  rc.worker.join();                        // the worker folds what is still in the inbox before it leaves
  adopt_published(pool);
  pool->recal.reset();
  return ODMA_OK;
}

int odma_pool_snapshot(const odma_pool_t* pool, int32_t max_n, int32_t* n_live, int32_t* req_id,
                       int32_t* arena, int64_t* offset, int32_t* cap, int32_t* len, int32_t* boundaries) {
  if (!pool || max_n < 0) {
    set_error("odma_pool_snapshot: invalid argument");
    return ODMA_INVALID_ARG;
  }
  int32_t k = 0, total = 0;
  for (int32_t rid = 0; rid < pool->cfg.max_requests; ++rid) {
    const Request& r = pool->req[rid];
    if (r.arena < 0) continue;
    ++total;
    if (k < max_n) {
      if (req_id) req_id[k] = rid;
      if (arena) arena[k] = r.arena;
      if (offset) offset[k] = r.off;
      if (cap) cap[k] = r.cap;
      if (len) len[k] = r.len;
      ++k;
    }
  }
  if (n_live) *n_live = total;
  if (boundaries) std::memcpy(boundaries, pool->boundaries.data(), sizeof(int32_t) * pool->boundaries.size());
  return ODMA_OK;
}

int odma_pool_free_extents(const odma_pool_t* pool, int32_t arena, int32_t max_n, int32_t* n_out,
                           int64_t* start, int64_t* size) {
  if (!pool || arena < 0 || arena > 1 || max_n < 0) {
    set_error("odma_pool_free_extents: invalid argument");
    return ODMA_INVALID_ARG;
  }
  const auto& fl = pool->arenas[arena].free_list;
  if (n_out) *n_out = (int32_t)fl.size();
  for (int32_t i = 0; i < max_n && i < (int32_t)fl.size(); ++i) {
    if (start) start[i] = fl[i].start;
    if (size) size[i] = fl[i].size;
  }
  return ODMA_OK;
}

int odma_pool_stats(const odma_pool_t* pool, odma_pool_stats_t* out) {
  if (!pool || !out) {
    set_error("odma_pool_stats: null argument");
    return ODMA_INVALID_ARG;
  }
  *out = pool->stats;
  out->boundary_epoch = pool->boundary_epoch;
  out->main_free = pool->arenas[0].free_tokens();
  out->safety_free = pool->arenas[1].free_tokens();
  return ODMA_OK;
}

int odma_pool_lookup(const odma_pool_t* pool, int32_t n, const int32_t* req_id, int64_t* offset,
                     int32_t* len, int32_t* cap) {
  if (!pool || n < 0 || (n > 0 && !req_id)) {
    set_error("odma_pool_lookup: null argument");
    return ODMA_INVALID_ARG;
  }
  for (int32_t i = 0; i < n; ++i) {
    int32_t rid = req_id[i];
    if (rid < 0 || rid >= pool->cfg.max_requests || pool->req[rid].arena < 0) {
      set_error("odma_pool_lookup: unknown request id");
      return ODMA_UNKNOWN_REQ;
    }
    const Request& r = pool->req[rid];
    if (offset) offset[i] = r.off;
    if (len) len[i] = r.len;
    if (cap) cap[i] = r.cap;
  }
  return ODMA_OK;
}

int odma_pool_tune(odma_pool_t* pool, int32_t knob, int32_t value) {
  if (!pool) {
    set_error("odma_pool_tune: null pool");
    return ODMA_INVALID_ARG;
  }
  switch (knob) {
    case ODMA_TUNE_WAVES_PER_CU:
      if (value < 0 || value > 64) break;
      pool->waves_per_cu = value;
      return ODMA_OK;
    case ODMA_TUNE_ITEMS_PER_WAVE:
      if (value < 4 || value > 256) break;
      pool->items_per_wave_x16 = value;
      return ODMA_OK;
    case ODMA_TUNE_MIN_CHUNK:
      if (value < 64 || value % 64) break;
      pool->min_chunk = value;
      return ODMA_OK;
    case ODMA_TUNE_WAVES_PER_WG:
      if (value != 0 && value != 4 && value != 8) break;
      pool->waves_per_wg = value;
      return ODMA_OK;
    case ODMA_TUNE_ODD_XCD_WEIGHT:
      if (value < 128 || value > 512) break;
      pool->odd_xcd_weight = value;
      return ODMA_OK;
    case ODMA_TUNE_LATE_WAVE_WEIGHT:
      if (value < 128 || value > 512) break;
      pool->late_wave_weight = value;
      return ODMA_OK;
    case ODMA_TUNE_FUSE_REDUCE:
      if (value != 0 && value != 1) break;
      pool->fuse_reduce = value;
      return ODMA_OK;
    case ODMA_TUNE_PREFILL_COLUMN_TILES:
      if (value != 0 && value != 2 && value != 4) break;
      pool->prefill_ct = value;
      return ODMA_OK;
    case ODMA_TUNE_PIPELINE_DEPTH:
      if (value != 2 && value != 3) break;
      pool->pipeline_depth = value;
      return ODMA_OK;
    default:
      break;
  }
  set_error("odma_pool_tune: unknown knob or value out of range");
  return ODMA_INVALID_ARG;
}

int odma_migrate_finish(odma_pool_t* pool, int32_t n, const int32_t* req_id, int32_t* status) {
  if (!pool || n < 0 || (n > 0 && !req_id)) {
    set_error("odma_migrate_finish: null argument");
    return ODMA_INVALID_ARG;
  }
  int first_err = ODMA_OK;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t rid = req_id[i];
    int st = ODMA_OK;
    if (rid < 0 || rid >= pool->cfg.max_requests || pool->req[rid].arena < 0 || pool->req[rid].held_arena < 0) {
      st = ODMA_UNKNOWN_REQ;
    } else {
      Request& r = pool->req[rid];
      pool->arenas[r.held_arena].release(r.held_off, r.held_cap);
      r.held_arena = -1;
      r.held_off = 0;
      r.held_cap = 0;
    }
    if (status) status[i] = st;
    if (st != ODMA_OK && first_err == ODMA_OK) first_err = st;
  }
  if (first_err != ODMA_OK) set_error("odma_migrate_finish: request not live or without a held source slab");
  return first_err;
}

int odma_migrate(odma_pool_t* pool, int32_t req_id, void* stream, int64_t* new_offset, int32_t* new_cap) {
  if (!pool) {
    set_error("odma_migrate: null pool");
    return ODMA_INVALID_ARG;
  }
  int64_t new_off = -1;
  int rc = migrate_begin(pool, req_id, &new_off);
  if (rc) return rc;
  const Request& r = pool->req[req_id];
  if (pool->cfg.k_pool && pool->cfg.v_pool && r.len > 0) {
    // one sequential copy per (layer, KV head, K|V): whole blocks covering len tokens
    const int64_t block_bytes = (int64_t)ODMA_BLOCK_TOKENS * pool->cfg.head_dim * pool->elem_bytes;
    const int64_t src = (r.off / ODMA_BLOCK_TOKENS) * block_bytes, dst = (new_off / ODMA_BLOCK_TOKENS) * block_bytes;
    const int64_t n_bytes = (int64_t)((r.len + ODMA_BLOCK_TOKENS - 1) / ODMA_BLOCK_TOKENS) * block_bytes;
    rc = migrate_copy ? migrate_copy(pool, 1, &src, &dst, &n_bytes, stream) : ODMA_HIP_ERROR;
    if (rc) {
      if (!migrate_copy) set_error("odma_migrate: this build of the library has no device half");
      migrate_abort(pool, new_off);
      return rc;
    }
  }
  migrate_commit(pool, req_id, new_off, false);
  if (new_offset) *new_offset = new_off;
  if (new_cap) *new_cap = pool->cfg.large_cap;
  return ODMA_OK;
}

int odma_migrate_batch(odma_pool_t* pool, int32_t n, const int32_t* req_id, uint32_t flags, void* stream,
                       int64_t* new_offset, int32_t* new_cap, int32_t* status) {
  if (!pool || n < 0 || (n > 0 && (!req_id || !new_offset || !new_cap || !status)) ||
      (flags & ~ODMA_MIGRATE_DEFER_RELEASE)) {
    set_error("odma_migrate_batch: invalid argument");
    return ODMA_INVALID_ARG;
  }
  const bool device = pool->cfg.k_pool && pool->cfg.v_pool;
  if (device && !migrate_copy) {
    set_error("odma_migrate_batch: this build of the library has no device half");
    return ODMA_HIP_ERROR;
  }
  const int64_t block_bytes = (int64_t)ODMA_BLOCK_TOKENS * pool->cfg.head_dim * pool->elem_bytes;
  std::vector<int64_t> src, dst, nb;
  int first_err = ODMA_OK;
  // Bookkeeping request by request in array order (sources live in the main arena, destinations in the safety
  // arena, so the order of releases cannot change a reservation); then the copies of all of them together.
  for (int32_t i = 0; i < n; ++i) {
    int64_t new_off = -1;
    const int rc = migrate_begin(pool, req_id[i], &new_off);
    status[i] = rc;
    new_offset[i] = rc == ODMA_OK ? new_off : -1;
    new_cap[i] = rc == ODMA_OK ? pool->cfg.large_cap : 0;
    if (rc != ODMA_OK) {
      if (first_err == ODMA_OK) first_err = rc;
      continue;
    }
    const Request& r = pool->req[req_id[i]];
    if (r.len > 0) {
      src.push_back((r.off / ODMA_BLOCK_TOKENS) * block_bytes);
      dst.push_back((new_off / ODMA_BLOCK_TOKENS) * block_bytes);
      nb.push_back((int64_t)((r.len + ODMA_BLOCK_TOKENS - 1) / ODMA_BLOCK_TOKENS) * block_bytes);
    }
    migrate_commit(pool, req_id[i], new_off, (flags & ODMA_MIGRATE_DEFER_RELEASE) != 0);
  }
  if (device && !src.empty()) {
    const int rc = migrate_copy(pool, (int32_t)src.size(), src.data(), dst.data(), nb.data(), stream);
    if (rc) return rc;                                       // bookkeeping has moved, data may not have: fatal
  }
  if (first_err != ODMA_OK) set_error("odma_migrate_batch: at least one request was not migrated; see status[]");
  return first_err;
}

int odma_pool_decode_kernel(const odma_pool_t* pool) { return pool ? pool->decode_kernel : ODMA_INVALID_ARG; }

int odma_stream_plan_ranges(int32_t total_tiles, int32_t n_waves, int32_t waves_per_wg, int32_t min_tiles,
                            int32_t odd_xcd_weight, int32_t late_wave_weight, int32_t* start, int32_t* waves_used) {
  if (total_tiles < 0 || n_waves <= 0 || (waves_per_wg != 4 && waves_per_wg != 8) || n_waves % waves_per_wg ||
      min_tiles < 1 || odd_xcd_weight < 128 || odd_xcd_weight > 512 || late_wave_weight < 128 ||
      late_wave_weight > 512 || !start) {
    set_error("odma_stream_plan_ranges: invalid argument");
    return ODMA_INVALID_ARG;
  }
  const odma_plan::StreamShares s =
      odma_plan::stream_shares(total_tiles, n_waves, waves_per_wg, min_tiles, odd_xcd_weight, late_wave_weight);
  for (int32_t w = 0; w <= n_waves; ++w) start[w] = s.start(w);
  if (waves_used) *waves_used = s.used;
  return ODMA_OK;
}

}  // extern "C"

// ---- migration bookkeeping -----------------------------------------------------------
namespace odma {

MigrateCopyFn migrate_copy = nullptr;      // installed by the device half when the library has one

// Reserves the Large-Bucket slab and rewrites the record; the caller enqueues the copy
// between `begin` and `commit` so that a HIP failure can roll back.
int migrate_begin(odma_pool* pool, int32_t rid, int64_t* new_off) {
  if (rid < 0 || rid >= pool->cfg.max_requests || pool->req[rid].arena < 0) {
    set_error("odma_migrate: unknown request id");
    return ODMA_UNKNOWN_REQ;
  }
  Request& r = pool->req[rid];
  if (r.arena == ODMA_ARENA_SAFETY) {
    set_error("odma_migrate: request already in the Large Bucket (reached large_cap)");
    return ODMA_OVERFLOW;
  }
  int64_t got = pool->arenas[ODMA_ARENA_SAFETY].reserve(pool->cfg.large_cap);
  if (got < 0) {
    pool->stats.nomem++;
    set_error("odma_migrate: safety arena exhausted");
    return ODMA_NOMEM;
  }
  *new_off = got;
  return ODMA_OK;
}

void migrate_abort(odma_pool* pool, int64_t new_off) {
  pool->arenas[ODMA_ARENA_SAFETY].release(new_off, pool->cfg.large_cap);
}

void migrate_commit(odma_pool* pool, int32_t rid, int64_t new_off, bool defer_release) {
  Request& r = pool->req[rid];
  if (defer_release) {
    r.held_arena = r.arena;
    r.held_off = r.off;
    r.held_cap = r.cap;
  } else {
    pool->arenas[r.arena].release(r.off, r.cap);
  }
  pool->stats.live_reserved += pool->cfg.large_cap - r.cap;
  r.left_behind += r.cap;
  pool->layout_gen++;
  r.arena = ODMA_ARENA_SAFETY;
  r.off = new_off;
  r.cap = pool->cfg.large_cap;
  pool->stats.migrations++;
}

}  // namespace odma
