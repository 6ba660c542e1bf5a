// C ABI of libpat.so: argument checks, plan lifetime, upload, and kernel launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <system_error>
#include <thread>
#include <vector>

#include "pat_common.hip.h"

namespace pat {
int build_plan(const pat_batch_desc &b, const pat_plan_opts &o, pat_plan_s &pl);
int advance_plan(pat_plan_s &pl, const int32_t *new_kv_lens, const int32_t *block_tables, int32_t W);
void refresh_view(pat_plan_s &pl);
bool tile_available(int id);
hipError_t launch_forward(int dtype, const FwdArgs &a, int n_entries, hipStream_t s);
hipError_t launch_forward_stream(int dtype, const FwdArgs &a, int n_workgroups, hipStream_t s);
hipError_t launch_merge(int dtype, const MergeArgs &a, hipStream_t s);
}  // namespace pat

using namespace pat;

// Debug aid: device buffer for per-workgroup timeline records of the next forward launches.
static unsigned long long *g_trace_buf = nullptr;
static size_t g_trace_records = 0;
// Debug aid: polls a workgroup spends on a claimed merge task before it leaves it to the last arriver.
static int g_spin_limit = 4096;

extern "C" {

int pat_debug_set_trace(void *device_buf, size_t bytes)
{
    if (device_buf && (bytes < 64 || reinterpret_cast<uintptr_t>(device_buf) % 8 != 0))
        return PAT_ERR_INVALID_ARG;
    g_trace_buf = static_cast<unsigned long long *>(device_buf);
    g_trace_records = device_buf ? bytes / 64 : 0;
    return PAT_OK;
}

int pat_debug_set_spin_limit(int polls)
{
    g_spin_limit = polls < 0 ? 4096 : polls;
    return PAT_OK;
}

int pat_plan(const pat_batch_desc *batch, const pat_plan_opts *opts, pat_plan_t **out_plan)
{
    if (!batch || !out_plan) return PAT_ERR_INVALID_ARG;
    pat_plan_opts o;
    std::memset(&o, 0, sizeof o);
    o.force_tile = -1;
    if (opts) o = *opts;
    pat_plan_s *pl = new (std::nothrow) pat_plan_s();
    if (!pl) return PAT_ERR_OUT_OF_MEMORY;
    int rc;
    try {
        rc = build_plan(*batch, o, *pl);
    } catch (const std::bad_alloc &) {
        rc = PAT_ERR_OUT_OF_MEMORY;
    } catch (...) {
        rc = PAT_ERR_INVALID_ARG;
    }
    if (rc != PAT_OK) {
        delete pl;
        return rc;
    }
    *out_plan = pl;
    return PAT_OK;
}

void pat_plan_destroy(pat_plan_t *plan)
{
    if (!plan) return;
    // the stream and events of a two-kernel launch (created by pat_plan_upload)
    if (plan->ev_fork) (void)hipEventDestroy(static_cast<hipEvent_t>(plan->ev_fork));
    if (plan->ev_join) (void)hipEventDestroy(static_cast<hipEvent_t>(plan->ev_join));
    if (plan->side_stream) (void)hipStreamDestroy(static_cast<hipStream_t>(plan->side_stream));
    delete plan;
}

// ---- planning on a worker thread ------------------------------------------------------------
struct pat_plan_job_s {
    pat_batch_desc batch;
    pat_plan_opts opts;
    bool have_opts = false;
    std::vector<int32_t> block_tables, kv_lens, node_parent, node_num_pages, req_leaf_node;
    std::thread worker;
    pat_plan_t *plan = nullptr;
    int status = PAT_ERR_INVALID_ARG;
};

int pat_plan_start(const pat_batch_desc *batch, const pat_plan_opts *opts, pat_plan_job_t **out_job)
{
    if (!batch || !out_job) return PAT_ERR_INVALID_ARG;
    if (batch->num_requests < 1 || batch->max_pages_per_req < 1 || !batch->block_tables ||
        !batch->kv_lens)
        return PAT_ERR_INVALID_ARG;
    if (batch->num_nodes > 0 && (!batch->node_parent || !batch->node_num_pages || !batch->req_leaf_node))
        return PAT_ERR_INVALID_ARG;
    try {
        std::unique_ptr<pat_plan_job_s> job(new pat_plan_job_s());
        job->batch = *batch;
        const size_t B = (size_t)batch->num_requests;
        job->block_tables.assign(batch->block_tables, batch->block_tables + B * batch->max_pages_per_req);
        job->kv_lens.assign(batch->kv_lens, batch->kv_lens + B);
        job->batch.block_tables = job->block_tables.data();
        job->batch.kv_lens = job->kv_lens.data();
        if (batch->num_nodes > 0) {
            job->node_parent.assign(batch->node_parent, batch->node_parent + batch->num_nodes);
            job->node_num_pages.assign(batch->node_num_pages, batch->node_num_pages + batch->num_nodes);
            job->req_leaf_node.assign(batch->req_leaf_node, batch->req_leaf_node + B);
            job->batch.node_parent = job->node_parent.data();
            job->batch.node_num_pages = job->node_num_pages.data();
            job->batch.req_leaf_node = job->req_leaf_node.data();
        }
        if (opts) {
            job->opts = *opts;
            job->have_opts = true;
        }
        pat_plan_job_s *j = job.get();
        j->worker = std::thread([j] {
            j->status = pat_plan(&j->batch, j->have_opts ? &j->opts : nullptr, &j->plan);
        });
        *out_job = job.release();
        return PAT_OK;
    } catch (const std::bad_alloc &) {
        return PAT_ERR_OUT_OF_MEMORY;
    } catch (const std::system_error &) {
        return PAT_ERR_OUT_OF_MEMORY;                       // no thread to be had
    }
}

int pat_plan_finish(pat_plan_job_t *job, pat_plan_t **out_plan)
{
    if (!job) return PAT_ERR_INVALID_ARG;
    if (job->worker.joinable()) job->worker.join();
    const int rc = job->status;
    if (rc == PAT_OK && out_plan) {
        *out_plan = job->plan;
    } else if (job->plan) {
        pat_plan_destroy(job->plan);                        // nobody takes it
    }
    delete job;
    return (rc == PAT_OK && !out_plan) ? PAT_ERR_INVALID_ARG : rc;
}

int pat_plan_get_stats(const pat_plan_t *plan, pat_plan_stats *stats)
{
    if (!plan || !stats) return PAT_ERR_INVALID_ARG;
    *stats = plan->stats;
    return PAT_OK;
}

int pat_plan_export(const pat_plan_t *plan, pat_plan_view *v)
{
    if (!plan || !v) return PAT_ERR_INVALID_ARG;
    try {
        // after pat_plan_advance(); two threads may export one plan at the same time
        pat_plan_t *mut = const_cast<pat_plan_t *>(plan);
        std::lock_guard<std::mutex> lock(mut->view_mutex);
        pat::refresh_view(*mut);
    } catch (const std::bad_alloc &) {
        return PAT_ERR_OUT_OF_MEMORY;
    }
    v->num_items = plan->stats.num_items;
    v->num_entries = plan->stats.num_entries;
    v->num_requests = plan->B;
    v->num_slots = plan->stats.num_slots;
    v->item_req_off = plan->item_req_off.data();
    v->item_req_ids = plan->item_req_ids.data();
    v->item_req_slot = plan->item_req_slot.data();
    v->item_page_off = plan->item_page_off.data();
    v->item_page_ids = plan->item_page_ids.data();
    v->item_page_start = plan->item_page_start.data();
    v->item_kv_len = plan->item_kv_len.data();
    v->req_slot_off = plan->req_slot_off.data();
    v->req_slot_ids = plan->req_slot_ids.data();
    v->entry_item = plan->entry_item.data();
    v->entry_row_begin = plan->entry_row_begin.data();
    v->entry_num_rows = plan->entry_num_rows.data();
    v->entry_tile = plan->entry_tile.data();
    v->entry_heads_per_wg = plan->entry_heads_per_wg.data();
    return PAT_OK;
}

int pat_plan_advance(pat_plan_t *plan, const int32_t *new_kv_lens, const int32_t *block_tables,
                     int32_t max_pages_per_req)
{
    if (!plan || !new_kv_lens || !block_tables || max_pages_per_req < 1) return PAT_ERR_INVALID_ARG;
    try {
        const int rc = pat::advance_plan(*plan, new_kv_lens, block_tables, max_pages_per_req);
        if (rc == PAT_OK) plan->device_buf = nullptr;           // the device copy is out of date
        return rc;
    } catch (const std::bad_alloc &) {
        return PAT_ERR_OUT_OF_MEMORY;
    }
}

int pat_plan_upload(pat_plan_t *plan, void *device_buf, size_t device_bytes, void *stream)
{
    if (!plan || !device_buf) return PAT_ERR_INVALID_ARG;
    if (device_bytes < plan->layout.total) return PAT_ERR_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(device_buf) % 256 != 0) return PAT_ERR_INVALID_ARG;
    hipError_t e = hipMemcpyAsync(device_buf, plan->staging.data(), plan->layout.total,
                                  hipMemcpyHostToDevice, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return PAT_ERR_HIP;
    if (plan->dual && !plan->side_stream) {
        // a stream of the plan's own (default priority) and the two events of the fork and join
        hipStream_t st = nullptr;
        hipEvent_t ef = nullptr, ej = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&ef, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ej, hipEventDisableTiming) != hipSuccess) {
            if (ef) (void)hipEventDestroy(ef);
            if (ej) (void)hipEventDestroy(ej);
            if (st) (void)hipStreamDestroy(st);
            return PAT_ERR_HIP;
        }
        plan->side_stream = st;
        plan->ev_fork = ef;
        plan->ev_join = ej;
    }
    plan->device_buf = device_buf;
    return PAT_OK;
}

int pat_num_tiles(void) { return NUM_TILES; }

int pat_tile_info(int tile_id, int *m, int *n)
{
    if (tile_id < 0 || tile_id >= NUM_TILES || !m || !n) return PAT_ERR_INVALID_ARG;
    *m = tile_info(tile_id).m;
    *n = tile_info(tile_id).n;
    return tile_available(tile_id) ? PAT_OK : PAT_ERR_UNSUPPORTED;
}

static int check_ws(const pat_plan_t *plan, const void *workspace, size_t workspace_bytes)
{
    if (!plan) return PAT_ERR_INVALID_ARG;
    if (!plan->device_buf) return PAT_ERR_PLAN_NOT_UPLOADED;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return PAT_ERR_INVALID_ARG;
    if (workspace_bytes < (size_t)plan->stats.workspace_bytes) return PAT_ERR_WORKSPACE_TOO_SMALL;
    return PAT_OK;
}

int pat_forward(const pat_plan_t *plan, const void *q, const void *k_pool, const void *v_pool,
                int64_t kv_stride_page, int64_t kv_stride_token, int64_t kv_stride_head,
                float softmax_scale, void *out, float *lse, void *workspace,
                size_t workspace_bytes, void *stream)
{
    // the packed tiles take the row maximum before scaling: the scale must keep the order
    if (!std::isfinite(softmax_scale) || !(softmax_scale > 0.f)) return PAT_ERR_INVALID_ARG;
    int rc = check_ws(plan, workspace, workspace_bytes);
    if (rc != PAT_OK) return rc;
    if (!q || !k_pool || !v_pool || !out) return PAT_ERR_INVALID_ARG;
    // 16-byte loads need every row start aligned: strides multiples of 8 elements
    if (kv_stride_page <= 0 || kv_stride_token <= 0 || kv_stride_head <= 0 ||
        kv_stride_page % 8 || kv_stride_token % 8 || kv_stride_head % 8)
        return PAT_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) |
         reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(out)) % 16 != 0)
        return PAT_ERR_INVALID_ARG;
    const unsigned char *dev = static_cast<const unsigned char *>(plan->device_buf);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    FwdArgs a;
    a.req_ids = reinterpret_cast<const int32_t *>(dev + plan->layout.req_ids);
    a.req_slot = reinterpret_cast<const int32_t *>(dev + plan->layout.req_slot);
    a.page_ids = reinterpret_cast<const int32_t *>(dev + plan->layout.page_ids);
    a.q = static_cast<const uint16_t *>(q);
    a.k_pool = static_cast<const uint16_t *>(k_pool);
    a.v_pool = static_cast<const uint16_t *>(v_pool);
    a.stride_page = kv_stride_page;
    a.stride_token = kv_stride_token;
    a.stride_head = kv_stride_head;
    a.out = static_cast<uint16_t *>(out);
    a.lse = lse;
    a.part_o = reinterpret_cast<float *>(ws + plan->ws_part_o);
    a.part_lse = reinterpret_cast<float *>(ws + plan->ws_part_lse);
    a.scale = softmax_scale;
    a.Hq = plan->Hq;
    a.Hkv = plan->Hkv;
    a.G = plan->Hq / plan->Hkv;
    a.trace = (g_trace_buf && g_trace_records >= (size_t)plan->stats.num_workgroups)
                  ? g_trace_buf : nullptr;
    hipStream_t s = static_cast<hipStream_t>(stream);
    a.units = reinterpret_cast<const DevUnit *>(dev + plan->layout.units);
    a.n_units = (int32_t)plan->units.size();
    a.queue_begin = plan->queue_begin;
    a.queue_workers = plan->queue_workers;
    a.queue_ctr = reinterpret_cast<int32_t *>(const_cast<unsigned char *>(dev) + plan->layout.queue_ctr);
    a.fuse_mode = plan->fuse_mode;
    a.n_merge = plan->stats.num_merge_requests;
    a.spin_limit = g_spin_limit;
    a.req_midx = reinterpret_cast<const int32_t *>(dev + plan->layout.req_midx);
    a.merge_rec = reinterpret_cast<const int32_t *>(dev + plan->layout.merge_rec);
    a.req_slot_ids = reinterpret_cast<const int32_t *>(dev + plan->layout.req_slot_ids);
    a.merge_state = reinterpret_cast<int32_t *>(const_cast<unsigned char *>(dev) + plan->layout.merge_state);
    a.workers = nullptr;
    a.wave_items = reinterpret_cast<const DevWaveItem *>(dev + plan->layout.wave_items);
    a.unit_base = 0;
    if (plan->dual) {
        // packed tiles on the caller's stream, 16-row tiles on the plan's own, side by side
        const int n_packed = plan->stream_begin, n_stream = (int)plan->units.size() - plan->stream_begin;
        hipStream_t side = static_cast<hipStream_t>(plan->side_stream);
        hipEvent_t fork = static_cast<hipEvent_t>(plan->ev_fork), join = static_cast<hipEvent_t>(plan->ev_join);
        if (n_stream > 0 && n_packed > 0) {
            if (hipEventRecord(fork, s) != hipSuccess || hipStreamWaitEvent(side, fork, 0) != hipSuccess)
                return PAT_ERR_HIP;
            if (launch_forward(plan->dtype, a, n_packed, s) != hipSuccess) return PAT_ERR_HIP;
            a.unit_base = n_packed;
            if (launch_forward_stream(plan->dtype, a, n_stream, side) != hipSuccess) return PAT_ERR_HIP;
            if (hipEventRecord(join, side) != hipSuccess || hipStreamWaitEvent(s, join, 0) != hipSuccess)
                return PAT_ERR_HIP;
        } else if (n_stream > 0) {
            if (launch_forward_stream(plan->dtype, a, n_stream, s) != hipSuccess) return PAT_ERR_HIP;
        } else if (launch_forward(plan->dtype, a, n_packed, s) != hipSuccess) {
            return PAT_ERR_HIP;
        }
        return PAT_OK;
    }
    int n_workgroups = plan->queue_begin + plan->queue_workers;
    if (!plan->workers.empty()) {
        a.workers = reinterpret_cast<const DevWorker *>(dev + plan->layout.workers);
        n_workgroups = (int)plan->workers.size();
    }
    if (launch_forward(plan->dtype, a, n_workgroups, s) != hipSuccess)
        return PAT_ERR_HIP;
    return PAT_OK;
}

int pat_merge(const pat_plan_t *plan, void *out, float *lse, const void *workspace,
              size_t workspace_bytes, void *stream)
{
    int rc = check_ws(plan, workspace, workspace_bytes);
    if (rc != PAT_OK) return rc;
    if (!out) return PAT_ERR_INVALID_ARG;
    const unsigned char *dev = static_cast<const unsigned char *>(plan->device_buf);
    const unsigned char *ws = static_cast<const unsigned char *>(workspace);
    MergeArgs m;
    m.merge_rec = reinterpret_cast<const int32_t *>(dev + plan->layout.merge_rec);
    m.req_slot_ids = reinterpret_cast<const int32_t *>(dev + plan->layout.req_slot_ids);
    m.part_o = reinterpret_cast<const float *>(ws + plan->ws_part_o);
    m.part_lse = reinterpret_cast<const float *>(ws + plan->ws_part_lse);
    m.out = static_cast<uint16_t *>(out);
    m.lse = lse;
    m.n_merge = plan->stats.num_merge_requests;
    m.Hq = plan->Hq;
    m.long_lists = plan->req_slot_ids.size() >= 8 * plan->merge_req.size();
    if (launch_merge(plan->dtype, m, static_cast<hipStream_t>(stream)) != hipSuccess)
        return PAT_ERR_HIP;
    return PAT_OK;
}

int pat_decode_attention(const pat_plan_t *plan, const void *q, const void *k_pool,
                         const void *v_pool, int64_t kv_stride_page, int64_t kv_stride_token,
                         int64_t kv_stride_head, float softmax_scale, void *out, float *lse,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = pat_forward(plan, q, k_pool, v_pool, kv_stride_page, kv_stride_token,
                         kv_stride_head, softmax_scale, out, lse, workspace, workspace_bytes,
                         stream);
    if (rc != PAT_OK) return rc;
    if (plan->fuse_mode) return PAT_OK;                 // the forward launch has merged
    return pat_merge(plan, out, lse, workspace, workspace_bytes, stream);
}

// ---- the same step for callers that cannot allocate device memory -------------------------------
// The workspace is a file-scope device array.  Its name is only a host-side handle: the address the
// kernels are given comes from hipGetSymbolAddress, once per device (every GPU holds its own copy).
static __device__ __align__(256) unsigned char scratch[PAT_STATIC_WORKSPACE_BYTES];
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64] = {nullptr};

static int static_workspace(void **ptr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PAT_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PAT_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return PAT_OK;
}

int pat_decode_attention_static_ws(const pat_plan_t *plan, const void *q, const void *k_pool,
                                   const void *v_pool, int64_t kv_stride_page,
                                   int64_t kv_stride_token, int64_t kv_stride_head,
                                   float softmax_scale, void *out, float *lse, void *stream)
{
    if (!plan) return PAT_ERR_INVALID_ARG;
    if ((size_t)plan->stats.workspace_bytes > (size_t)PAT_STATIC_WORKSPACE_BYTES)
        return PAT_ERR_WORKSPACE_TOO_SMALL;
    void *ws = nullptr;
    const int rc = static_workspace(&ws);
    if (rc != PAT_OK) return rc;
    // every partial the merge reads is written by this call's forward first: nothing to clear
    return pat_decode_attention(plan, q, k_pool, v_pool, kv_stride_page, kv_stride_token,
                                kv_stride_head, softmax_scale, out, lse, ws,
                                PAT_STATIC_WORKSPACE_BYTES, stream);
}

const char *pat_strerror(int status)
{
    switch (status) {
    case PAT_OK: return "ok";
    case PAT_ERR_INVALID_ARG: return "invalid argument";
    case PAT_ERR_BAD_PAGE_ID: return "block table names a page id outside the pool";
    case PAT_ERR_BAD_KV_LEN: return "kv_len < 1 or longer than the block-table row";
    case PAT_ERR_UNSUPPORTED: return "unsupported head_dim, page_size, dtype or tile";
    case PAT_ERR_WORKSPACE_TOO_SMALL: return "device buffer too small";
    case PAT_ERR_PLAN_NOT_UPLOADED: return "plan has not been uploaded";
    case PAT_ERR_HIP: return "HIP runtime call failed";
    case PAT_ERR_OUT_OF_MEMORY: return "host allocation failed";
    case PAT_ERR_BAD_TREE: return "explicit prefix tree disagrees with the block tables";
    case PAT_ERR_PLAN_STALE: return "the change needs a new plan";
    default: return "unknown status";
    }
}

const char *pat_version(void) { return "pat-mi355x 0.1"; }

}  // extern "C"
