/*
 * libodma -- C ABI of the MI355X (gfx950) decode hot path behind ODMA, the
 * on-demand contiguous KV-cache allocation strategy of "ODMA: On-Demand Memory
 * Allocation Strategy for LLM Serving on LPDDR-Class Accelerators".
 *
 * The paper's pipeline (Section III-A): predict a generation length, reserve a
 * matched CONTIGUOUS block of KV memory, decode while streaming that block, fall
 * back to the Large Bucket (safety pool) on high uncertainty or overflow
 * (Section III-D), and re-derive bucket boundaries from an online histogram of
 * realized lengths (Section III-C, Eq. 2).  This library holds
 *   - the host allocator and bookkeeping (assign / advance / migrate / release /
 *     recalibrate), deterministic and integer-exact, and
 *   - the device kernels that touch the KV pool: per-step KV append, batched GQA
 *     decode attention over each request's slab (split-K online softmax plus a
 *     cross-split reduction), and the migration copy.
 *
 * Conventions
 *   Pointers   Every argument marked DEVICE is a device pointer; everything else
 *              is host memory.  The caller owns every device byte (pools,
 *              workspace, q, out, offset/length arrays); the library owns only the
 *              host-side odma_pool_t and never allocates or frees device memory.
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *              Device calls are asynchronous and stream-ordered.
 *   Errors     Every call returns ODMA_OK or a negative code; batch calls also fill
 *              a per-request status array.  A failed request leaves the pool
 *              unchanged for that request.  Nothing throws, aborts or exits across
 *              the ABI.  odma_last_error() returns a thread-local message.
 *   Threads    A pool is externally synchronized (one caller at a time), with one exception: while the
 *              background recalibrator runs, odma_report_completions and odma_recalibrator_drain may be
 *              called from any thread beside the one that drives the pool.
 *   Tokens     All sizes, offsets, capacities and lengths are in tokens.  The main
 *              arena is [0, main_tokens), the safety arena (Large Bucket) is
 *              [main_tokens, main_tokens + safety_tokens): one address space, so a
 *              single offset indexes the device pool.
 *
 * Device pool format (library-defined; write it with odma_append_kv, read it with
 * odma_decode_attention or odma_gather_kv -- do not index it directly)
 *   k_pool and v_pool each hold n_layers * n_kv_heads * pool_tokens * head_dim
 *   elements, pool_tokens = main_tokens + safety_tokens, arranged as
 *       [layer][kv_head][block][16 tokens x head_dim elements]
 *   A block is 16 consecutive token slots of one KV head; a slab is a run of
 *   consecutive blocks, so slab offsets and capacities are multiples of 16.
 *   Inside a K block element (t, d) sits at  ((d / x) * 16 + t) * x + d % x,
 *   x = 16 bytes / element size (8 for bf16, 4 for fp32): 16-byte pieces of 16
 *   tokens are adjacent, which is the operand order of the gfx950 16x16x32 MFMA.
 *   Inside a V block element (t, d) sits at
 *       (((d / 32) * 4 + t / 4) * 16 + d % 16) * 8 + ((d / 16) % 2) * 4 + t % 4
 *   (V is transposed inside the block: four consecutive tokens of one channel are
 *   adjacent, the order in which the P*V product consumes them).
 *   The paged variant uses the same blocks, found through a block table instead of
 *   offset / 16 + t / 16.
 *   ODMA_FP8 pools (head_dim 128): a block is 16 tokens x 128 bytes; K element (t, d) sits at byte
 *       (((d / 64) * 4 + (d / 8) % 4) * 16 + t) * 16 + ((d / 32) % 2) * 8 + d % 8
 *   and V element (t, d) at byte
 *       ((d / 64) * 64 + (t / 4) * 16 + d % 16) * 16 + ((d / 16) % 4) * 4 + t % 4
 *   (the operand order of the gfx950 16x16x32 fp8 MFMA).
 */
#ifndef ODMA_H
#define ODMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ODMA_OK            0
#define ODMA_INVALID_ARG  (-1)
#define ODMA_NOMEM        (-2)   /* arena exhausted */
#define ODMA_OVERFLOW     (-3)   /* past capacity without migration, or past large_cap */
#define ODMA_UNKNOWN_REQ  (-4)   /* unknown, duplicate or already released request id */
#define ODMA_HIP_ERROR    (-5)   /* HIP runtime error; text in odma_last_error() */

#define ODMA_F32   0
#define ODMA_BF16  1
#define ODMA_FP8   2     /* OCP E4M3 (1-4-3, bias 7, no infinities, 0x7f/0xff = NaN): K and V storage only; q stays bf16 */

#define ODMA_ARENA_MAIN    0
#define ODMA_ARENA_SAFETY  1

#define ODMA_BLOCK_TOKENS  16    /* tokens per pool block == page size of the paged variant */

/* decode kernel choice */
#define ODMA_KERNEL_AUTO   0     /* MFMA kernel when the shape allows, else the VALU kernel */
#define ODMA_KERNEL_VALU   1     /* fp32 vector-ALU kernel: any dtype, head_dim % 32 == 0 */
#define ODMA_KERNEL_MFMA   2     /* matrix-core kernel: bf16 storage with head_dim 128 or 64, fp8 storage with head_dim 128; group <= 16 */

/* odma_decode_attention flags */
#define ODMA_REUSE_PLAN    1     /* caller asserts that n, lengths, offsets and the choice between offsets and a block
                                    table are what the previous planning call on this pool saw (the 28 layers of one
                                    step): skip re-planning.  The matrix-core plan bakes the slab bases in, so the
                                    library drops the flag by itself, and plans again, whenever it knows the assertion
                                    cannot hold: n differs, contiguous/paged differs, a request was assigned, released
                                    or migrated since, or a launch-shape knob changed.  Changed lengths, or offsets
                                    edited by the caller, it cannot see. */
#define ODMA_SKIP_REDUCE   2     /* kernel timing only: no cross-split reduction (neither the launch nor the in-kernel
                                    merge), so outputs of requests split over several chunks are NOT valid */

typedef struct odma_pool odma_pool_t;   /* opaque, host side */

typedef struct odma_pool_config {
  int32_t n_layers;
  int32_t n_q_heads;        /* Hq; consecutive groups of Hq/Hkv query heads share a KV head */
  int32_t n_kv_heads;       /* Hkv */
  int32_t head_dim;         /* D, multiple of 32, <= 256 */
  int32_t kv_dtype;         /* ODMA_F32 | ODMA_BF16: storage of q, K and V; ODMA_FP8: K and V in E4M3 (one byte per
                               element, real value = stored value x k_scale / v_scale), q in bf16 */
  int32_t out_dtype;        /* ODMA_F32 | ODMA_BF16 */
  int32_t align_tokens;     /* slab alignment and histogram bin width; multiple of 16 */
  int32_t large_cap;        /* capacity of one Large-Bucket slab (L_max), multiple of align_tokens */
  int64_t main_tokens;      /* main arena size, multiple of align_tokens */
  int64_t safety_tokens;    /* safety arena size, multiple of align_tokens */
  int32_t max_requests;     /* request ids are 0 .. max_requests-1 */
  int32_t n_buckets;        /* B (the paper uses 4, Section III-C) */
  const int32_t* boundaries;    /* initial b_1 < ... < b_B, multiples of align_tokens, <= large_cap */
  const int32_t* quantile_num;  /* p_i = num/den for Eq. 2; NULL -> {1/2,4/5,19/20,99/100} for B = 4, */
  const int32_t* quantile_den;  /*   {1/2,9/10,99/100} for B = 3 (the paper does not print its levels) */
  int32_t window;           /* sliding window of realized lengths (paper: 10000) */
  int32_t decode_kernel;    /* ODMA_KERNEL_* */
  double  gamma;            /* inflation weight, paper: 0.2 (Section III-B) */
  double  tau;              /* routing threshold, paper: 0.8 */
  float   sm_scale;         /* softmax scale; 0 -> 1/sqrt(head_dim) */
  int32_t max_splits;       /* upper bound on (request, chunk) work items the plan may create beyond
                               one per request; 0 -> 8192.  Sizes the workspace. */
  float   k_scale, v_scale; /* ODMA_FP8 only: de-quantisation factors of the K and V pools; 0 -> 1 */
  void*   k_pool;           /* DEVICE, caller-owned, see "Device pool format" */
  void*   v_pool;           /* DEVICE */
  void*   workspace;        /* DEVICE, at least odma_workspace_bytes() bytes, 256-byte aligned */
  size_t  workspace_bytes;
} odma_pool_config_t;

typedef struct odma_pool_stats {
  int64_t live_requests, live_tokens, live_reserved;   /* now */
  int64_t main_free, safety_free;                       /* free tokens per arena */
  int64_t done_requests, done_actual, done_reserved;    /* released so far: sum len, sum cap at release */
  int64_t done_reserved_both;                           /* ... counting also slabs left behind by migration */
  int64_t migrations, nomem, recalibrations;
  int64_t boundary_epoch;                               /* background recalibrator: epoch of the boundaries in use */
} odma_pool_stats_t;

/* Bytes of device workspace the decode kernels of Sections III-A / V-B need for this configuration (plan,
 * work list and split-K partial results).  Pointers inside cfg are ignored.  0 on
 * an invalid configuration. */
size_t odma_workspace_bytes(const odma_pool_config_t* cfg);

/* Creates the host-side pool over caller-owned device memory (the Allocator of Section III-A,
 * which keeps the free lists of one device).  Works without a GPU when k_pool,
 * v_pool and workspace are NULL (allocator-only use; device calls then fail with
 * ODMA_INVALID_ARG). */
int odma_pool_create(const odma_pool_config_t* cfg, odma_pool_t** out);
/* Ends the pool's life cycle (Section III-E): stops the background recalibrator if one runs and frees the host
 * record.  Device memory stays the caller's.  NULL is accepted. */
int odma_pool_destroy(odma_pool_t* pool);

/* L' = ceil(pred_len * (1 + gamma*u)) in IEEE double (Section III-B). */
int64_t odma_inflate(const odma_pool_t* pool, int32_t pred_len, float u);

/* Admission (Sections III-A, III-B, III-D).  For request i, in array order:
 *   need = prompt_len[i] + (uncertainty ? inflate(pred_len[i], uncertainty[i]) : pred_len[i]);
 *   u > tau (strict) or need > b_B  -> Large Bucket: cap = large_cap, safety arena, bucket = B;
 *   else bucket = min{ j : b_j >= need }, cap = b_j, main arena;
 *   reserve = lowest-address free extent with size >= cap (first fit), low end taken.
 * Outputs per request: bucket (-1 on failure), offset (-1), cap (0), status
 * (ODMA_OK | INVALID_ARG | UNKNOWN_REQ for an id already live | OVERFLOW when need >
 * large_cap | NOMEM).  uncertainty, prompt_len and boundaries may be NULL (u = 0 and no
 * inflation; prompt 0; the pool's current boundaries).  boundaries passed here are
 * validated, used for this call only and never touch live requests (Section IV-C).
 * Returns ODMA_OK or the first per-request error. */
int odma_assign(odma_pool_t* pool, int32_t n, const int32_t* req_id, const int32_t* pred_len,
                const float* uncertainty, const int32_t* prompt_len,
                const int32_t* boundaries, int32_t n_boundaries,
                int32_t* bucket, int64_t* offset, int32_t* cap, int32_t* status);

/* Completion (Section III-E `release`): returns each slab to its arena, coalescing
 * with free neighbours, and adds the request to the utilization totals (Section V).
 * status may be NULL. */
int odma_release(odma_pool_t* pool, int32_t n, const int32_t* req_id, int32_t* status);

/* Bookkeeping of newly generated tokens: len += n_new[i] (n_new NULL -> 1) unless that
 * exceeds the slab capacity, in which case overflow[i] = 1 and len is unchanged
 * (Section III-D: the trigger of reactive migration).  status may be NULL. */
int odma_advance(odma_pool_t* pool, int32_t n, const int32_t* req_id, const int32_t* n_new,
                 int32_t* overflow, int32_t* status);

/* Reactive migration (Section III-D, allocate-and-copy of Section IV-C): reserves a
 * Large-Bucket slab, enqueues on `stream` one sequential copy of the request's len
 * tokens (rounded up to whole blocks) for every layer, K and V, releases the source
 * slab and updates the record.  The source may be reused immediately by later calls
 * because any write into it is enqueued on the same stream after the copy.
 * Errors: UNKNOWN_REQ; OVERFLOW if the request already sits in the safety arena (it
 * has reached L_max); NOMEM if the safety arena is full (request untouched). */
int odma_migrate(odma_pool_t* pool, int32_t req_id, void* stream,
                 int64_t* new_offset, int32_t* new_cap);

/* Adaptive Bucket Manager (Section III-C, Eq. 2): pushes n realized lengths (clamped to
 * [1, large_cap]) into the sliding window, evicting the oldest, then sets
 *   b_i = (j_i + 1) * align,  j_i = first histogram bin whose cumulative count reaches
 *   k_i = max(1, ceil(p_i * n_window))   (integer arithmetic on p_i = num/den),
 * forces b_i >= b_{i-1} + align, then clamps from the top so that b_B <= large_cap.
 * An empty window leaves the boundaries unchanged.  Writes n_buckets values. */
int odma_recalibrate(odma_pool_t* pool, int32_t n, const int32_t* realized_len,
                     int32_t* boundaries_out);

/* Batched migration: odma_migrate for n requests in array order, with all their copies in as few
 * launches as possible (one launch covers every layer, K and V, of up to 16 requests).  A request
 * that cannot be migrated gets its error in status[i] and is left untouched; the others proceed;
 * the return value is the first error (or ODMA_OK).  new_offset/new_cap/status: host arrays of n.
 *   flags = ODMA_MIGRATE_DEFER_RELEASE: the source slabs stay reserved until odma_migrate_finish.
 *   This is what lets the copy run on a stream of its own beside the decode step of the other
 *   requests (Section III-D calls migration rare and off the common path): enqueue the batch on a
 *   copy stream, keep decoding the non-migrating requests on the compute stream, make the compute
 *   stream wait for the copy (an event) before the migrated requests rejoin with their new offsets,
 *   then call odma_migrate_finish, which releases the sources.  Without the flag the sources are
 *   released at once and same-stream ordering protects them, as in odma_migrate.
 * odma_release of a request whose source is still held releases the source as well. */
#define ODMA_MIGRATE_DEFER_RELEASE 1u
int odma_migrate_batch(odma_pool_t* pool, int32_t n, const int32_t* req_id, uint32_t flags, void* stream,
                       int64_t* new_offset, int32_t* new_cap, int32_t* status);
/* Releases the source slabs kept by ODMA_MIGRATE_DEFER_RELEASE.  status (nullable) per request:
 * ODMA_OK, or ODMA_UNKNOWN_REQ if the request is not live or holds no source. */
int odma_migrate_finish(odma_pool_t* pool, int32_t n, const int32_t* req_id, int32_t* status);

/* Background recalibration (Sections III-E and IV-C: the histogram is maintained off the
 * critical path and the boundaries are swapped in without stopping admission).
 *   odma_recalibrator_start    starts a thread owned by the pool.  It folds reported completions
 *                              into the sliding window in the order they were reported and after
 *                              every `refresh_every` of them recomputes the boundaries (same rule as
 *                              odma_recalibrate) and publishes them with an epoch number 1, 2, ...
 *                              While it runs, odma_recalibrate is refused (the thread owns the window).
 *   odma_report_completions    hands realized total lengths to the thread; returns at once.
 *   odma_assign                adopts the newest published set at the start of each call, reading it
 *                              through a sequence lock (no mutex on the admission path); the epoch in
 *                              use is odma_pool_stats_t.boundary_epoch.  Which epoch a given call sees
 *                              depends on timing; the set belonging to an epoch does not.
 *   odma_recalibrator_drain    blocks until everything reported so far is folded; *epoch (nullable)
 *                              receives the newest published epoch.  For tests and deterministic replays.
 *   odma_recalibrator_stop     folds what is pending, joins the thread, adopts the last set.
 * Apart from these three calls the pool stays externally synchronized, as before. */
int odma_recalibrator_start(odma_pool_t* pool, int32_t refresh_every);
int odma_report_completions(odma_pool_t* pool, int32_t n, const int32_t* realized_len);
int odma_recalibrator_drain(odma_pool_t* pool, int64_t* epoch);
int odma_recalibrator_stop(odma_pool_t* pool);

/* Live requests in increasing id order, at most max_n of them (n_live receives the full count); arrays may be
 * NULL.  boundaries (nullable) receives the n_buckets boundaries in use (Section III-C). */
int odma_pool_snapshot(const odma_pool_t* pool, int32_t max_n, int32_t* n_live,
                       int32_t* req_id, int32_t* arena, int64_t* offset, int32_t* cap,
                       int32_t* len, int32_t* boundaries /* n_buckets */);
/* Free extents of one arena in address order: at most max_n (start, size) pairs. */
int odma_pool_free_extents(const odma_pool_t* pool, int32_t arena, int32_t max_n,
                           int32_t* n_out, int64_t* start, int64_t* size);
int odma_pool_stats(const odma_pool_t* pool, odma_pool_stats_t* out);
/* Host copy of (offset, len) for a batch of live requests, to build the device arrays. */
int odma_pool_lookup(const odma_pool_t* pool, int32_t n, const int32_t* req_id,
                     int64_t* offset, int32_t* len, int32_t* cap);

/* Per-step KV append (the growing per-request cache of Section II-A, written into the
 * contiguous reservation of Section I-C).  For request i the n_new[i] rows
 * k_new[src_start[i] + j] / v_new[...] (j < n_new[i], each row [Hkv][D] in kv_dtype)
 * are written at token positions[i] + j of its slab (offsets[i]) or, when block_table
 * is given, of its block list block_table[i*bt_stride + ...].
 *   offsets     DEVICE int64[n]   slab base (ignored when block_table != NULL)
 *   positions   DEVICE int32[n]   first token index to write (the current length)
 *   n_new       DEVICE int32[n] or NULL (one row each; then src_start may be NULL: row i)
 *   src_start   DEVICE int64[n] or NULL
 *   max_new     host upper bound on n_new[i] (sizes the launch); 1 when n_new is NULL
 *   k_new,v_new DEVICE
 * n must not exceed max_requests (ODMA_INVALID_ARG).  The library does not check capacity here (it cannot see
 * device arrays): call odma_advance first and migrate flagged requests. */
int odma_append_kv(odma_pool_t* pool, int32_t layer, int32_t n,
                   const int64_t* offsets, const int32_t* positions,
                   const int32_t* n_new, const int64_t* src_start, int32_t max_new,
                   const int32_t* block_table, int32_t bt_stride,
                   const void* k_new, const void* v_new, void* stream);

/* Batched GQA decode attention (the streaming read that contiguous allocation exists
 * to serve, Sections III-A and V-B).  For request r, query head h, g = h / (Hq/Hkv):
 *   s_t = sm_scale * <q[r,h,:], K_r[t,g,:]>,  p = softmax_t(s),  out[r,h,:] = sum_t p_t V_r[t,g,:]
 * over all t < lengths[r]; fp32 accumulation; a request with length 0 yields zeros.
 *   q        DEVICE [n][Hq][D] kv_dtype        out  DEVICE [n][Hq][D] out_dtype
 *   offsets  DEVICE int64[n]                   lengths DEVICE int32[n]
 *   block_table DEVICE int32[n][bt_stride] or NULL (contiguous slabs)
 * Launches a plan kernel (unless ODMA_REUSE_PLAN), the split-K attention kernel and
 * the cross-split reduction on `stream`, using the pool's workspace; calls on one
 * pool must therefore not overlap on different streams. */
int odma_decode_attention(odma_pool_t* pool, int32_t layer, int32_t n,
                          const void* q, const int64_t* offsets, const int32_t* lengths,
                          const int32_t* block_table, int32_t bt_stride,
                          void* out, uint32_t flags, void* stream);

/* Fused decode step: odma_append_kv of one row per request at position lengths[r]-1 followed
 * by odma_decode_attention over lengths[r] tokens, in one pass over the pool (the wave that
 * streams a request's last block patches the new row in and writes it to the pool).
 * lengths are the lengths AFTER the append and must be >= 1 (a request with length 0 is
 * skipped and yields zeros).  k_new, v_new: DEVICE [n][Hkv][D] kv_dtype.  Other arguments as
 * for odma_decode_attention.  One launch on the matrix-core kernel; on the vector-ALU kernel the
 * row append and the attention are launched one after the other.  Capacity is the caller's business (odma_advance / odma_migrate). */
int odma_decode_step(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, const void* k_new,
                     const void* v_new, const int64_t* offsets, const int32_t* lengths,
                     const int32_t* block_table, int32_t bt_stride, void* out, uint32_t flags,
                     void* stream);

/* odma_decode_attention for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels and bit-identical
 * results, but the plan records, arrival counters and partial states live in a static device array inside the library
 * (ODMA_STATIC_SCRATCH_BYTES, held on every GPU the library runs on until the process ends) instead of the pool's
 * workspace, which may be NULL.  The call allocates nothing and calls no allocating routine.
 *   Limits   matrix-core pools only; n <= ODMA_STATIC_MAX_REQUESTS; the launch shape may use at most
 *            ODMA_STATIC_MAX_WORKGROUPS work-groups (the default on MI355X uses 256); the query-head count must fit
 *            the array (up to 60 heads).  Beyond a limit: ODMA_INVALID_ARG with the reason in odma_last_error().
 *   flags    0 or ODMA_REUSE_PLAN (honoured only if the previous call on this GPU's array planned for this pool in
 *            its present state; otherwise the call plans again).
 *   Sharing  all pools and all calls on one GPU share that GPU's array, and it keeps the last call's contents; the
 *            plan kernel clears the counters that must start at zero.  Calls that overlap on one GPU (two streams,
 *            two threads) race: serialise them. */
#define ODMA_STATIC_SCRATCH_BYTES   (16u << 20)
#define ODMA_STATIC_MAX_REQUESTS    1024
#define ODMA_STATIC_MAX_WORKGROUPS  256
int odma_decode_attention_static(odma_pool_t* pool, int32_t layer, int32_t n,
                                 const void* q, const int64_t* offsets, const int32_t* lengths,
                                 const int32_t* block_table, int32_t bt_stride,
                                 void* out, uint32_t flags, void* stream);

/* Prefill (chunk) attention over the same slabs: the last n_q[r] of the lengths[r] tokens of
 * request r each carry a query (their K/V rows are already in the pool: odma_append_kv first),
 * and query j, at position lengths[r] - n_q[r] + j, attends causally to tokens 0 .. that
 * position of its slab -- the prompt phase that fills the reservation of Section III-A before
 * decoding starts; a whole prompt is n_q = length, a later chunk of a long prompt n_q < length.
 * Same definition per query as odma_decode_attention; bf16 or fp8 pools with head_dim 128 only
 * (ODMA_INVALID_ARG otherwise); q is bf16 in both cases.
 *   q, out     DEVICE [total_q][Hq][D] bf16 / out_dtype: the query tokens of all requests, request
 *              r's rows at q_start[r] .. q_start[r] + n_q[r] - 1 (rows need not be ordered or dense)
 *   total_q    host: rows of q and out; rows at or past it are never read or written
 *   q_start    DEVICE int64[n]        n_q  DEVICE int32[n] (0: nothing to do; clamped to lengths[r])
 *   offsets, lengths, block_table, bt_stride as for odma_decode_attention (lengths include the chunk)
 * Launches a plan kernel and the attention kernel on `stream`, using the pool's workspace. */
int odma_prefill_attention(odma_pool_t* pool, int32_t layer, int32_t n, const void* q, int64_t total_q,
                           const int64_t* q_start, const int32_t* n_q, const int64_t* offsets,
                           const int32_t* lengths, const int32_t* block_table, int32_t bt_stride,
                           void* out, void* stream);

/* Export of one request's KV in plain row-major order: k_out, v_out DEVICE
 * [length][Hkv][D] in kv_dtype.  block_row (DEVICE int32[]) selects the paged layout. */
int odma_gather_kv(odma_pool_t* pool, int32_t layer, int64_t offset, int32_t length,
                   const int32_t* block_row, void* k_out, void* v_out, void* stream);

/* Measurement aid, not part of the method: reads `bytes` bytes (a multiple of 16) of the DEVICE
 * buffer `buf` once, with a chip-wide linear sweep (the access pattern that reads fastest on
 * MI355X), asynchronously on `stream`.  Timing it gives the read rate the part actually sustains,
 * to set beside the published HBM peak.  `sink` (DEVICE, 4 bytes) keeps the reads alive; it is
 * written only if a checksum hits one particular value.  Needs no pool. */
int odma_stream_read_probe(const void* buf, size_t bytes, void* sink, void* stream);

/* Measurement aid, not part of the method: what the scattered fetches of a paged pool cost a pure read,
 * the effect Sections I-C and II-A argue from.  In the launch shape of the attention kernel (4 waves
 * per compute unit, each streaming an equal share) step s reads the 4 KiB block table[s] of k_plane
 * and of v_plane (DEVICE, each at least (max table entry + 1) * 4096 bytes; DEVICE int32 table[n_steps],
 * entries >= 0), double buffered with the block id fetched one step ahead.  table = 0, 1, 2, ... reads
 * one contiguous slab; a permutation reads what a paged pool with 4 KiB blocks looks like.  Asynchronous
 * on `stream`; `sink` as above.  The caller guarantees that every table entry lies inside the planes. */
int odma_block_read_probe(const void* k_plane, const void* v_plane, const int32_t* table, int64_t n_steps,
                          void* sink, void* stream);

/* Launch-shape knobs for experiments and benchmarks; defaults suit MI355X.  Returns
 * ODMA_INVALID_ARG for an unknown knob or a value outside its range. */
#define ODMA_TUNE_WAVES_PER_CU     1   /* decode waves launched per compute unit, 1..64; 0 = default (MFMA kernel: 4 = one per
                                          SIMD; VALU kernel: 8) */
#define ODMA_TUNE_ITEMS_PER_WAVE   2   /* VALU kernel: work items aimed at per wave, in sixteenths, 4..256 (default 32 = 2.0) */
#define ODMA_TUNE_MIN_CHUNK        3   /* smallest range a wave is given, in tokens, multiple of 64 (default 64) */
#define ODMA_TUNE_PIPELINE_DEPTH   4   /* register tile buffers per wave in the MFMA kernel: 2 or 3 (default 2) */
#define ODMA_TUNE_WAVES_PER_WG     5   /* MFMA kernel work-group size in waves: 4 or 8; 0 = default (4) */
#define ODMA_TUNE_ODD_XCD_WEIGHT   6   /* MFMA kernel: tile share of work-groups on odd XCDs relative to even
                                          ones, in 1/256 (128..512, default 256 = equal) */
#define ODMA_TUNE_LATE_WAVE_WEIGHT 7   /* MFMA kernel, 8-wave work-groups: tile share of waves 4..7 (the second wave on
                                          each SIMD) relative to waves 0..3, in 1/256 (128..512, default 256) */
#define ODMA_TUNE_FUSE_REDUCE      8   /* MFMA kernel: 1 (default) merges segments cut between work-groups inside the attention
                                          launch (last work-group to arrive), 0 in a reduction launch of its own */
#define ODMA_TUNE_PREFILL_COLUMN_TILES 9 /* prefill kernel: 16-column tiles per wave.  2 (0 = default): 128-column work items, two
                                          work-groups per CU.  4: 256-column items, one work-group per CU (more reuse per
                                          K/V byte, measured slower on every prompt mix tried) */
int odma_pool_tune(odma_pool_t* pool, int32_t knob, int32_t value);

/* Test aid, host only, needs no pool: the tile ranges the matrix-core plan gives its waves.  The batch's tiles
 * (16-token blocks, counted over requests and KV heads) form one stream; wave w of n_waves (a multiple of
 * waves_per_wg = 4 or 8) streams [start[w], start[w + 1]).  min_tiles: fewest tiles per wave before fewer waves
 * are used; weights as for ODMA_TUNE_ODD_XCD_WEIGHT / _LATE_WAVE_WEIGHT.  start: host int32[n_waves + 1];
 * waves_used: nullable.  Guarantee that the attention kernel depends on: among the used waves the empty ranges
 * come first (no empty range lies between two ranges that hold tiles). */
int odma_stream_plan_ranges(int32_t total_tiles, int32_t n_waves, int32_t waves_per_wg, int32_t min_tiles,
                            int32_t odd_xcd_weight, int32_t late_wave_weight, int32_t* start, int32_t* waves_used);

/* Names the decode kernel the pool resolved to (ODMA_KERNEL_VALU or _MFMA). */
int odma_pool_decode_kernel(const odma_pool_t* pool);

const char* odma_last_error(void);
const char* odma_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ODMA_H */
