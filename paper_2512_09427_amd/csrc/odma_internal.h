// Internal definitions shared by the host allocator (odma_host.cpp) and the device
// entry points (odma_device.hip).  Not part of the ABI.
#pragma once

#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstddef>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "odma.h"
#include "plan_types.h"

namespace odma {

struct Extent {
  int64_t start, size;
};

// Address-ordered first-fit extent list with coalescing (the reading of the paper's
// "free lists", Section III-E, that stays well defined when boundaries move).
struct Arena {
  int64_t base = 0, size = 0;
  std::vector<Extent> free_list;
  void init(int64_t b, int64_t s);
  int64_t reserve(int64_t cap);            // returns start or -1
  void release(int64_t off, int64_t cap);
  int64_t free_tokens() const;
};

struct Request {
  int32_t arena = -1;                      // -1: not live
  int64_t off = 0;
  int32_t cap = 0, len = 0;
  int64_t left_behind = 0;                 // capacity of slabs released by migration
  int32_t held_arena = -1;                 // source slab of a migration whose release was deferred
  int64_t held_off = 0;
  int32_t held_cap = 0;
};

// Sliding window of realized lengths and its histogram with align-wide bins; boundaries are the
// upper edges of the bins where the cumulative count reaches the quantile ranks (Section III-C).
struct Calibrator {
  std::vector<int32_t> ring, qnum, qden;
  size_t head = 0, count = 0;
  std::vector<int64_t> hist;
  int32_t align = 16, large_cap = 0;
  void push(int32_t realized_len);
  bool compute(int32_t* b, int32_t n_buckets) const;   // false when the window is empty (b untouched)
};

// Background recalibration (Sections III-E, IV-C): a thread owned by the pool folds reported
// completions into the window and every `refresh` of them publishes new boundaries.  Readers
// (odma_assign) take the published set through a sequence lock: no mutex on the admission path.
struct Recalibrator {
  std::thread worker;
  std::mutex mu;                           // guards inbox, stop
  std::condition_variable wake, idle;
  std::vector<int32_t> inbox;
  bool stop = false;
  int32_t refresh = 0;
  int64_t reported = 0;                    // under mu
  std::atomic<int64_t> folded{0};          // completions the worker has folded into the window
  std::atomic<uint32_t> seq{0};            // even: pub_* stable; odd: being written
  std::atomic<int64_t> pub_epoch{0};
  std::atomic<int32_t> pub_b[64];          // n_buckets <= 64
};

// Device workspace carve-up (byte offsets from cfg.workspace); the record types it sizes are in plan_types.h.
struct WorkspaceLayout {
  size_t header = 0, req_info = 0, items = 0, waves = 0, red = 0, arrive = 0, part_ml = 0, part_o = 0, prefill = 0, total = 0;
  int64_t max_pairs = 0;
};

WorkspaceLayout workspace_layout(const odma_pool_config_t& cfg);
bool validate_config(const odma_pool_config_t& cfg, std::string* why);
int resolve_decode_kernel(const odma_pool_config_t& cfg);
void set_error(const std::string& msg);
// Copy of n byte runs (the same in every (layer, KV head) plane of K and of V), enqueued on `stream`; the device half
// of the library installs it when it is loaded.  A library built from the host half alone leaves it null: it serves
// pools without device memory (allocator-only use, sanitizer builds).
typedef int (*MigrateCopyFn)(odma_pool* pool, int32_t n, const int64_t* src_byte, const int64_t* dst_byte,
                             const int64_t* n_bytes, void* stream);
extern MigrateCopyFn migrate_copy;
int migrate_begin(odma_pool* pool, int32_t rid, int64_t* new_off);
void migrate_abort(odma_pool* pool, int64_t new_off);
void migrate_commit(odma_pool* pool, int32_t rid, int64_t new_off, bool defer_release);

}  // namespace odma

struct odma_pool {
  odma_pool_config_t cfg;
  std::vector<int32_t> boundaries;
  odma::Arena arenas[2];
  std::vector<odma::Request> req;
  odma::Calibrator calib;                  // used by odma_recalibrate, or by the worker while one runs
  std::unique_ptr<odma::Recalibrator> recal;
  int64_t boundary_epoch = 0;              // published epoch the current boundaries came from
  odma_pool_stats_t stats{};
  // device side
  odma::WorkspaceLayout ws;
  int decode_kernel = ODMA_KERNEL_VALU;
  int n_cu = 0;                            // filled on first device call
  int64_t pool_blocks = 0;                 // (main+safety)/16
  size_t elem_bytes = 2;
  // launch-shape knobs (odma_pool_tune)
  int waves_per_cu = 0;                    // 0: default (MFMA kernel 4 = one wave per SIMD; VALU kernel 8)
  int items_per_wave_x16 = 32;
  int min_chunk = 0;                       // 0: kernel default
  int waves_per_wg = 0;                    // MFMA kernel: waves that heal range cuts among themselves (4 or 8)
  int odd_xcd_weight = 256;                // share of a work-group on an odd XCD, in 1/256 of an even one's
  int late_wave_weight = 256;              // share of waves 4..7 of an 8-wave work-group, in 1/256 of waves 0..3
  int prefill_ct = 0;                      // prefill kernel: column tiles per wave (0: by mean chunk length, 2, 4)
  int fuse_reduce = 1;                     // MFMA kernel: 1 merges cut segments inside the attention launch, 0 in a launch of its own
  int pipeline_depth = 2;                  // register tile buffers per wave in the MFMA kernel (2 or 3)
  // What the plan in the workspace was made for.  A plan bakes in the slab bases (or the fact that a block table
  // is used) and the launch shape; ODMA_REUSE_PLAN is honoured only while all of these still hold, otherwise the
  // call plans again.  layout_gen counts every change of a request's slab (assign, release, migration).
  uint64_t layout_gen = 1;
  struct PlanStamp {
    uint64_t layout_gen = 0;               // 0: no plan yet
    int32_t n = -1, paged = -1, n_wg = 0, wpw = 0, q_min = 0, tile_tokens = 0, odd_w = 0, late_w = 0;
    uint64_t owner = 0;                    // serial of the pool that planned (the static scratch serves every pool)
  } plan_stamp;
  uint64_t serial = 0;                     // unique per pool ever created in this process
};
