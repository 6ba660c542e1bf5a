/*
 * pat.h -- C ABI of the prefix-aware decode-attention library for MI355X (gfx950).
 *
 * The library implements the pack -> forward -> merge paradigm of the paper
 * (sec. "Insight: Pack-forward-merge Paradigm"):
 *   pack    : pat_plan()              CPU, integers only.  Block table -> prefix forest ->
 *                                     TreeHeuristic (Algorithm 1) -> long-KV split -> tile
 *                                     selection -> schedule of work items.
 *   forward : pat_forward()           GPU.  One workgroup per (work item, KV head): partial
 *                                     attention with online softmax over the item's pages.
 *   merge   : pat_merge()             GPU.  Per (request, q head): log-sum-exp combination of
 *                                     the request's partial results.
 *   pat_decode_attention() = forward + merge on one stream.
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on the
 *     current device.  The caller owns every buffer it passes; the library owns only the
 *     opaque pat_plan_t and frees it in pat_plan_destroy().
 *   - Streams are passed as void* (a hipStream_t; NULL = the default stream).  GPU entry
 *     points only enqueue work and never synchronise; launch errors are returned, execution
 *     faults surface at the caller's next synchronisation.
 *   - Every function returns PAT_OK (0) or a negative pat_status.  No exceptions cross the ABI,
 *     nothing aborts, and output arguments are untouched on failure.
 *   - A plan is immutable after pat_plan_upload() and may serve any number of forward/merge
 *     calls (all layers and all decode steps until the block table changes -- the paper's
 *     lazy update, sec. "Pack Scheduler").  Calls that share one workspace must not overlap, and
 *     neither must forward calls that share one uploaded plan buffer: it holds two counters of
 *     the forward kernel's unit queue (zero between launches).
 */
#ifndef PAT_H_
#define PAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pat_plan_s pat_plan_t;

typedef enum {
    PAT_OK = 0,
    PAT_ERR_INVALID_ARG = -1,        /* NULL pointer, non-positive size, Hq % Hkv != 0 ...      */
    PAT_ERR_BAD_PAGE_ID = -2,        /* a referenced block-table entry is < 0 or >= num_pages   */
    PAT_ERR_BAD_KV_LEN = -3,         /* kv_len < 1 or more pages than max_pages_per_req         */
    PAT_ERR_UNSUPPORTED = -4,        /* head_dim != 128, page_size != 16, unknown dtype/tile    */
    PAT_ERR_WORKSPACE_TOO_SMALL = -5,
    PAT_ERR_PLAN_NOT_UPLOADED = -6,
    PAT_ERR_HIP = -7,                /* a HIP runtime call or kernel launch failed              */
    PAT_ERR_OUT_OF_MEMORY = -8,      /* host allocation failed                                  */
    PAT_ERR_BAD_TREE = -9,           /* explicit prefix tree disagrees with the block tables    */
    PAT_ERR_PLAN_STALE = -10         /* pat_plan_advance(): the change needs a new plan         */
} pat_status;

typedef enum { PAT_F16 = 0, PAT_BF16 = 1 } pat_dtype;

/* Packing mode.  PAT = Algorithm 1.  NAIVE_PER_NODE = one pack per tree node (the paper's
 * "naive" ablation, sec. "Ablation Study").  NO_SHARING = one pack per request over its whole
 * row: the one-query-per-workgroup baseline the speed-up is measured against. */
typedef enum {
    PAT_MODE_PAT = 0,
    PAT_MODE_NAIVE_PER_NODE = 1,
    PAT_MODE_NO_SHARING = 2
} pat_mode;

/* Long-KV split policy (sec. "Multi Kernel Forward", paragraph "Long KV Split").
 * MEAN   : the paper's rule -- packs longer than the mean pack length are cut into
 *          ceil(len/mean) page-aligned parts of (almost) equal page count, and into more
 *          while a part of several pages is still longer than the mean.
 * NONE   : no splitting.
 * TARGET : packs longer than split_target_tokens are cut into ceil(len/target) parts.
 * AUTO   : TARGET with a target derived from the batch and the device's CU count so that the
 *          launch holds several workgroups per CU (default). */
typedef enum {
    PAT_SPLIT_AUTO = 0,
    PAT_SPLIT_MEAN = 1,
    PAT_SPLIT_NONE = 2,
    PAT_SPLIT_TARGET = 3
} pat_split_policy;

/* Description of one decode batch.  All pointers: host memory, read during pat_plan() only. */
typedef struct {
    int32_t num_requests;            /* B >= 1                                                  */
    int32_t max_pages_per_req;       /* row pitch of block_tables                               */
    const int32_t *block_tables;     /* [B][max_pages_per_req] page ids; entries at or beyond   */
                                     /*   ceil(kv_len/page_size) of a row are ignored           */
    const int32_t *kv_lens;          /* [B] tokens per request, >= 1                            */
    int32_t page_size;               /* tokens per page; 16                                     */
    int32_t num_pages;               /* size of the page pool, for bounds checks                */
    int32_t num_q_heads;             /* Hq                                                      */
    int32_t num_kv_heads;            /* Hkv, divides Hq; q head h reads kv head h / (Hq/Hkv)    */
    int32_t head_dim;                /* 128                                                     */
    int32_t dtype;                   /* pat_dtype of q, K, V and out                            */
    /* Optional explicit prefix tree (sec. "Pack Scheduler", "Tree Structure Block Table").
     * num_nodes == 0 / NULL pointers: the forest is derived from identical leading page ids.
     * Otherwise node i has parent node_parent[i] (-1 = root; a parent precedes its children),
     * owns node_num_pages[i] consecutive block-table entries after its parent's, and request r
     * ends in node req_leaf_node[r].  Pages of a node with more than one request below it must
     * be identical in, and completely filled by, all of those requests, else PAT_ERR_BAD_TREE. */
    int32_t num_nodes;
    const int32_t *node_parent;
    const int32_t *node_num_pages;
    const int32_t *req_leaf_node;
} pat_batch_desc;

typedef struct {
    int32_t mode;                    /* pat_mode                                                */
    int32_t merge_factor;            /* child c merges into its parent unless                   */
                                     /*   merge_factor * s_c < len(blocks); 0 = the paper's 4   */
    int32_t split_policy;            /* pat_split_policy                                        */
    int32_t split_target_tokens;     /* PAT_SPLIT_TARGET only                                   */
    int32_t force_tile;              /* -1 = tile selector, else a tile id for every item       */
    int32_t num_cus;                 /* 0 = 256 (MI355X); used by PAT_SPLIT_AUTO                */
    int32_t tail_reserve_pages;      /* page slots kept free behind each request's own last     */
                                     /*   item for pat_plan_advance(): 0 = 16, negative = none  */
    int32_t model_ns[4];             /* run-time model of PAT_SPLIT_AUTO for one-round batches, */
                                     /*   ns: packed workgroup = [0] + [1] * tokens, 16-row     */
                                     /*   workgroup = [2] + [3] * tokens * KV heads; all 0 =    */
                                     /*   the built-in MI355X calibration                       */
    int32_t wave_kv_tokens;          /* 16-row packs of up to wave_max_tokens tokens are cut    */
                                     /*   into parts of at most this many tokens, each (part,   */
                                     /*   KV head) walked by ONE wavefront (tile n = 32).       */
                                     /*   0 = the planner's own rule (launches of nothing but   */
                                     /*   unshared requests of up to 384 tokens; 16-row packs   */
                                     /*   of up to 96 tokens beside anything); negative = never */
    int32_t wave_max_tokens;         /* 0 = 4 * wave_kv_tokens                                  */
    int32_t dual_launch;             /* forward as TWO kernels side by side (sec. "Multi-Stream */
                                     /*   Forward"): packed tiles as 512-thread workgroups on   */
                                     /*   the caller's stream, 16-row tiles as 256-thread       */
                                     /*   workgroups (one KV head each, two per CU) on a stream */
                                     /*   of the plan's own that forks from and joins the       */
                                     /*   caller's.  1 = on; 0 or -1 = off (measured slower on  */
                                     /*   MI355X, so never the planner's own choice)            */
    int32_t fused_merge;             /* merge inside the forward launch (no second kernel): a   */
                                     /*   per-(request, KV head) arrival counter tells the last */
                                     /*   workgroup to arrive to merge that request's partials; */
                                     /*   in launches of one round, workgroups that are done    */
                                     /*   claim requests and wait (bounded) for their partials. */
                                     /*   1 = on; 0 or -1 = off (measured slower than the merge */
                                     /*   kernel on MI355X, so never the planner's own choice)  */
    int32_t packed_min_tokens;       /* 17..32 rows over fewer tokens than this run as two      */
                                     /*   16-row blocks, not as one 64-row packed workgroup;    */
                                     /*   0 = the built-in MI355X crossover (48)                */
    int32_t reserved[1];             /* must be 0                                               */
} pat_plan_opts;

typedef struct {
    int32_t num_nodes;               /* nodes of the prefix forest, leaves included             */
    int32_t num_packs;               /* packs after TreeHeuristic, before splitting             */
    int32_t num_merged_children;     /* children packed by Scheme 2                             */
    int32_t num_items;               /* work items after long-KV split                          */
    int32_t num_entries;             /* (item, row block) units                                 */
    int32_t num_workgroups;          /* units of work of the forward launch                     */
    int32_t num_slots;               /* partial-result slots in the workspace                   */
    int32_t num_merge_requests;      /* requests with more than one partial                     */
    int64_t unique_kv_tokens;        /* sum of item kv_len = tokens read once by the forward    */
    int64_t total_kv_tokens;         /* sum of kv_lens = tokens a one-query-per-CTA kernel reads*/
    int64_t plan_device_bytes;       /* size pat_plan_upload() needs                            */
    int64_t workspace_bytes;         /* size forward/merge need                                 */
    int32_t num_wave_items;          /* (entry, KV head) items walked by one wavefront each;    */
                                     /*   num_workgroups counts them next to the workgroup-     */
                                     /*   level units (one timeline record each)                */
    int32_t num_workers;             /* persistent workgroups of a launch with such items, or 0 */
    int32_t fused_merge;             /* 0: forward then merge kernel; 1: the forward launch     */
                                     /*   merges (last arriver); 2: the same with claimed waits */
    int32_t pad0;
    int32_t tile_histogram[16];      /* entries per tile id                                     */
} pat_plan_stats;

/* Read-only host views of the schedule; valid until pat_plan_destroy().  Items are listed in
 * launch order.  Item i: requests item_req_ids[item_req_off[i] .. item_req_off[i+1]) (ascending),
 * which all hold pages item_page_ids[item_page_off[i] .. item_page_off[i+1]) at row positions
 * item_page_start[i] ..; item_kv_len[i] valid tokens (only the last page may be partial, and
 * then the item has one request).  item_req_slot runs parallel to item_req_ids: the partial
 * slot written for that (item, request), or -1 when the request has no other item and the
 * forward kernel writes its final output directly.  Request r merges slots
 * req_slot_ids[req_slot_off[r] .. req_slot_off[r+1]).  Entry e = (item entry_item[e], rows
 * entry_row_begin[e] .. + entry_num_rows[e]) with tile entry_tile[e]; a row is
 * (request position in item) * (Hq/Hkv) + (head within group).  An entry is launched as
 * ceil(Hkv / entry_heads_per_wg[e]) workgroups (packed tiles: 1 head each; 16-row tiles: 2,
 * or 1 where the device-aware split spreads a long pack over more CUs). */
typedef struct {
    int32_t num_items, num_entries, num_requests, num_slots;
    const int32_t *item_req_off, *item_req_ids, *item_req_slot;
    const int32_t *item_page_off, *item_page_ids, *item_page_start;
    const int32_t *item_kv_len;
    const int32_t *req_slot_off, *req_slot_ids;
    const int32_t *entry_item, *entry_row_begin, *entry_num_rows, *entry_tile;
    const int32_t *entry_heads_per_wg;
} pat_plan_view;

/* pack: prefix tree + block tables in, schedule out.  opts may be NULL (defaults).
 * On success *out_plan receives a new plan. */
int pat_plan(const pat_batch_desc *batch, const pat_plan_opts *opts, pat_plan_t **out_plan);
void pat_plan_destroy(pat_plan_t *plan);
int pat_plan_get_stats(const pat_plan_t *plan, pat_plan_stats *stats);
int pat_plan_export(const pat_plan_t *plan, pat_plan_view *view);

/* Planning off the critical path (sec. "Pack Scheduler": the scheduler runs on the CPU next to the
 * GPU's work of the previous step).  pat_plan_start() copies the batch description (block
 * tables, kv_lens, the optional tree: the caller's buffers are free again when it returns) and
 * plans on a worker thread of its own; pat_plan_finish() waits for that thread, hands over the
 * plan (or the planner's error status, with *out_plan untouched) and frees the job.  Every job
 * must be finished exactly once; out_plan == NULL discards the result (PAT_ERR_INVALID_ARG). */
typedef struct pat_plan_job_s pat_plan_job_t;
int pat_plan_start(const pat_batch_desc *batch, const pat_plan_opts *opts, pat_plan_job_t **out_job);
int pat_plan_finish(pat_plan_job_t *job, pat_plan_t **out_plan);

/* Lazy update (sec. "Pack Scheduler": the schedule is reused across decode steps and updated
 * only where the block table changed).  A decode step appends one token to every request: its
 * kv_len grows by one and, every page_size steps, one page id is appended to its row.
 * pat_plan_advance() brings the plan up to date in place when that is all that happened since
 * pat_plan() (or the previous advance):
 *   - new_kv_lens[r] >= the plan's kv_len of r, for every r;
 *   - the entries of row r below its old page count are unchanged (the caller's promise; the
 *     last one is checked), new page ids follow them and are inside the pool;
 *   - a request that grows ends in an item of its own (not in pages it shares to the very end
 *     with another request) and that item's reserve (pat_plan_opts.tail_reserve_pages) has room.
 * Otherwise nothing is changed and PAT_ERR_PLAN_STALE is returned: plan again.  Packs, splits
 * and tiles stay as planned (a request's last item simply gets longer), so plan again now and
 * then.  On success the host schedule and the staging image are current; call
 * pat_plan_upload() again (one copy) before the next forward.  Views from an earlier
 * pat_plan_export() are invalid afterwards. */
int pat_plan_advance(pat_plan_t *plan, const int32_t *new_kv_lens, const int32_t *block_tables,
                     int32_t max_pages_per_req);

/* Plan cache keyed by a fingerprint of the block table (sec. "Pack Scheduler": the schedule is
 * reused while the block table stays the same and updated lazily when it grows).
 * pat_plan_cache_get() hands out the plan for `batch` and says in *how (may be NULL) where it came
 * from: 1 = the same batch (same kv_lens, same used block-table entries, same heads, dtype and
 * options) was planned before: that plan, unchanged (its uploaded copy, if any, is still good);
 * 2 = a cached batch some decode steps later (no request shorter, old pages in place): that plan
 * brought up to date with pat_plan_advance() -- upload it again; 0 = planned anew (the least
 * recently used plan is destroyed when `capacity` plans are held).  The cache owns the plans: they
 * live until they are evicted or the cache is destroyed, and must not be passed to
 * pat_plan_destroy().  Not thread-safe. */
typedef struct pat_plan_cache_s pat_plan_cache_t;
int pat_plan_cache_create(int32_t capacity, pat_plan_cache_t **out_cache);
void pat_plan_cache_destroy(pat_plan_cache_t *cache);
int pat_plan_cache_get(pat_plan_cache_t *cache, const pat_batch_desc *batch, const pat_plan_opts *opts,
                       pat_plan_t **out_plan, int32_t *how);

/* Copy the schedule into caller-owned device memory (>= stats.plan_device_bytes, 256-byte
 * aligned) with hipMemcpyAsync on `stream`; the buffer must outlive every forward/merge call
 * made with this plan.  The host staging copy is pageable, so the call returns after the
 * copy has been handed to the runtime.
 * The image also holds the launch's counters (the unit queue's head, the fused merge's arrival
 * counts); every launch leaves them at zero for the next one.  A launch that did NOT run to its
 * end (an execution fault, a device reset, a process that was stopped inside it) can leave them
 * anywhere: after any failed or abandoned launch, upload the plan again before using it. */
int pat_plan_upload(pat_plan_t *plan, void *device_buf, size_t device_bytes, void *stream);

/* Tile shapes of the forward kernel family (sec. "Multi-tile Kernel"): m = query rows a
 * workgroup holds, n = KV tokens per pipeline stage of the workgroup.  Returns
 * PAT_ERR_INVALID_ARG for an unknown id.  pat_num_tiles() ids are valid. */
int pat_num_tiles(void);
int pat_tile_info(int tile_id, int *m, int *n);

/* forward (sec. "Multi-tile Kernel", sec. "Multi Kernel Forward"): for every work item and KV
 * head, S = scale * Q K^T over the item's tokens, online softmax, O = P V, fp32 accumulation.
 * Writes one fp32 partial (normalised O [d] and natural-log LSE) per (item, request, q head)
 * into the workspace, or the final out/lse directly for requests with a single item.  Plans with
 * the merge fused into this launch (pat_plan_stats.fused_merge != 0) also write the merged
 * out/lse of every other request; pat_merge() after it is then redundant (and harmless).
 *   q          device [B][Hq][d], dtype, contiguous
 *   k_pool     device; element (page, token, kv head, c) at
 *   v_pool       page*kv_stride_page + token*kv_stride_token + head*kv_stride_head + c
 *              (strides in elements; d contiguous; 16-byte aligned rows)
 *   softmax_scale  finite and > 0, else PAT_ERR_INVALID_ARG
 *   out        device [B][Hq][d], dtype
 *   lse        device [B][Hq] fp32, natural log of sum exp(scaled scores); may be NULL
 *   workspace  device, >= stats.workspace_bytes, 256-byte aligned                              */
int pat_forward(const pat_plan_t *plan, const void *q, const void *k_pool, const void *v_pool,
                int64_t kv_stride_page, int64_t kv_stride_token, int64_t kv_stride_head,
                float softmax_scale, void *out, float *lse, void *workspace,
                size_t workspace_bytes, void *stream);

/* merge (sec. "Output Merge"): for every request with more than one partial and every q head,
 * L = logsumexp_i LSE_i, out = sum_i exp(LSE_i - L) O_i, written in dtype; lse (may be NULL). */
int pat_merge(const pat_plan_t *plan, void *out, float *lse, const void *workspace,
              size_t workspace_bytes, void *stream);

/* forward + merge on `stream`. */
int pat_decode_attention(const pat_plan_t *plan, const void *q, const void *k_pool,
                         const void *v_pool, int64_t kv_stride_page, int64_t kv_stride_token,
                         int64_t kv_stride_head, float softmax_scale, void *out, float *lse,
                         void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops
 * and harnesses that forbid hipMalloc): pat_decode_attention() with the workspace taken from a
 * fixed array of PAT_STATIC_WORKSPACE_BYTES inside the library's device image (every GPU the
 * library runs on holds its own copy until the process ends).  q, pools, out, lse and the plan's
 * uploaded buffer are the caller's as before.  Calls no allocating routine.  A plan whose
 * stats.workspace_bytes exceeds the array is refused with PAT_ERR_WORKSPACE_TOO_SMALL and
 * nothing is launched.  All calls on one GPU share the array: calls that overlap on one GPU (two
 * streams, two threads) race; calls one after the other on one stream are fine, and nothing of
 * an earlier call is read (the forward stage writes every partial the merge stage reads). */
#define PAT_STATIC_WORKSPACE_BYTES (32u << 20)
int pat_decode_attention_static_ws(const pat_plan_t *plan, const void *q, const void *k_pool,
                                   const void *v_pool, int64_t kv_stride_page,
                                   int64_t kv_stride_token, int64_t kv_stride_head,
                                   float softmax_scale, void *out, float *lse, void *stream);

/* Debug aid (the analogue of the paper's per-SM CTA timelines, sec. "Ablation Study").  While a
 * device buffer is set, every pat_forward() whose launch has at most bytes/64 workgroups writes
 * one record of eight uint64 per workgroup, in launch order: start and end time on the GPU's
 * 100 MHz constant clock, (XCC_ID << 32 | HW_ID) of the wavefront that ran it,
 * (tile id << 32 | entry kv_len), and four intermediate marks, 0 where a tile does not take
 * one (0: first K/V tile has landed for 16-row tiles, first loads issued for packed tiles;
 * 1: first packed tile computed; 2: main loop done; 3: first loads issued for 16-row tiles,
 * first tile landed for packed tiles).  NULL switches it off (the default).  Process-wide;
 * not thread-safe. */
int pat_debug_set_trace(void *device_buf, size_t bytes);

/* Debug aid for the fused merge's claimed waits: the number of polls (about 0.3 us each) a
 * workgroup spends on a request whose partials are not complete before it leaves the request to
 * the last arriver.  0 makes every wait give up at once (the fallback path, for tests); negative
 * restores the default (4096).  Process-wide; not thread-safe. */
int pat_debug_set_spin_limit(int polls);

const char *pat_strerror(int status);
const char *pat_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PAT_H_ */
