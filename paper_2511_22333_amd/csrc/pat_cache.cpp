// Plan cache keyed by a fingerprint of the block table (sec. "Pack Scheduler", lazy update: the
// schedule is computed once and reused while the block table stays as it is, and brought up to
// date in place when decode steps only made requests longer).  Host only.
#include <cstring>
#include <list>
#include <new>
#include <vector>

#include "pat.h"

namespace {

struct Entry {
    uint64_t fingerprint = 0;
    pat_batch_desc desc{};                    // scalar fields only; pointers are not kept
    pat_plan_opts opts{};
    std::vector<int32_t> kv_lens;             // [B]
    std::vector<int32_t> row_off;             // [B + 1] into pages
    std::vector<int32_t> pages;               // the used entries of every block-table row
    std::vector<int32_t> tree;                // node_parent, node_num_pages, req_leaf_node (or empty)
    pat_plan_t *plan = nullptr;
};

inline void mix(uint64_t &h, uint64_t x)
{
    h ^= x;
    h *= 0x100000001b3ull;                    // FNV-1a over 64-bit words
}

// Everything the planner's result depends on, flattened.  Entries of a row beyond its page count
// are ignored by the planner and are not part of the key.
void flatten(const pat_batch_desc &b, Entry &e)
{
    const int32_t B = b.num_requests, P = b.page_size;
    e.desc = b;
    e.desc.block_tables = nullptr;
    e.desc.kv_lens = nullptr;
    e.desc.node_parent = e.desc.node_num_pages = e.desc.req_leaf_node = nullptr;
    e.desc.max_pages_per_req = 0;             // a wider table with the same used entries is the same batch
    e.kv_lens.assign(b.kv_lens, b.kv_lens + B);
    e.row_off.assign(1, 0);
    e.pages.clear();
    for (int32_t r = 0; r < B; ++r) {
        const int32_t n = (b.kv_lens[r] + P - 1) / P;
        const int32_t *row = b.block_tables + (int64_t)r * b.max_pages_per_req;
        e.pages.insert(e.pages.end(), row, row + n);
        e.row_off.push_back((int32_t)e.pages.size());
    }
    e.tree.clear();
    if (b.num_nodes > 0) {
        e.tree.insert(e.tree.end(), b.node_parent, b.node_parent + b.num_nodes);
        e.tree.insert(e.tree.end(), b.node_num_pages, b.node_num_pages + b.num_nodes);
        e.tree.insert(e.tree.end(), b.req_leaf_node, b.req_leaf_node + B);
    }
    uint64_t h = 0xcbf29ce484222325ull;
    const int32_t scal[] = {b.num_requests, b.page_size, b.num_pages, b.num_q_heads, b.num_kv_heads,
                            b.head_dim, b.dtype, b.num_nodes};
    for (int32_t x : scal) mix(h, (uint32_t)x);
    const int32_t *o = reinterpret_cast<const int32_t *>(&e.opts);
    for (size_t i = 0; i < sizeof(pat_plan_opts) / 4; ++i) mix(h, (uint32_t)o[i]);
    for (int32_t x : e.kv_lens) mix(h, (uint32_t)x);
    for (int32_t x : e.pages) mix(h, (uint32_t)x);
    for (int32_t x : e.tree) mix(h, (uint32_t)x);
    e.fingerprint = h;
}

// Field by field: the descriptor has padding, whose bytes a caller's copy need not define.
bool same_shape(const Entry &a, const Entry &b)
{
    const pat_batch_desc &x = a.desc, &y = b.desc;
    static_assert(sizeof(pat_plan_opts) % 4 == 0 && alignof(pat_plan_opts) == 4, "opts: int32 fields only");
    return x.num_requests == y.num_requests && x.page_size == y.page_size && x.num_pages == y.num_pages &&
           x.num_q_heads == y.num_q_heads && x.num_kv_heads == y.num_kv_heads && x.head_dim == y.head_dim &&
           x.dtype == y.dtype && x.num_nodes == y.num_nodes &&
           std::memcmp(&a.opts, &b.opts, sizeof a.opts) == 0 && a.tree == b.tree;
}

// `now` is `then` after decode steps: no request shorter, every old page still in its place.
bool is_successor(const Entry &then, const Entry &now)
{
    if (!same_shape(then, now) || !then.tree.empty()) return false;
    const size_t B = then.kv_lens.size();
    for (size_t r = 0; r < B; ++r) {
        if (now.kv_lens[r] < then.kv_lens[r]) return false;
        const int32_t n_old = then.row_off[r + 1] - then.row_off[r];
        if (now.row_off[r + 1] - now.row_off[r] < n_old) return false;
        if (std::memcmp(&then.pages[then.row_off[r]], &now.pages[now.row_off[r]], sizeof(int32_t) * (size_t)n_old))
            return false;
    }
    return true;
}

}  // namespace

struct pat_plan_cache_s {
    size_t capacity = 0;
    std::list<Entry> entries;                 // most recently used first
};

extern "C" {

int pat_plan_cache_create(int32_t capacity, pat_plan_cache_t **out_cache)
{
    if (capacity < 1 || !out_cache) return PAT_ERR_INVALID_ARG;
    pat_plan_cache_s *c = new (std::nothrow) pat_plan_cache_s();
    if (!c) return PAT_ERR_OUT_OF_MEMORY;
    c->capacity = (size_t)capacity;
    *out_cache = c;
    return PAT_OK;
}

void pat_plan_cache_destroy(pat_plan_cache_t *cache)
{
    if (!cache) return;
    for (Entry &e : cache->entries) pat_plan_destroy(e.plan);
    delete cache;
}

int pat_plan_cache_get(pat_plan_cache_t *cache, const pat_batch_desc *batch, const pat_plan_opts *opts,
                       pat_plan_t **out_plan, int32_t *how)
{
    if (!cache || !batch || !out_plan) return PAT_ERR_INVALID_ARG;
    if (batch->num_requests < 1 || batch->max_pages_per_req < 1 || batch->page_size < 1 ||
        !batch->block_tables || !batch->kv_lens)
        return PAT_ERR_INVALID_ARG;
    if (batch->num_nodes > 0 && (!batch->node_parent || !batch->node_num_pages || !batch->req_leaf_node))
        return PAT_ERR_INVALID_ARG;
    for (int32_t r = 0; r < batch->num_requests; ++r)     // the key is built from the used entries
        if (batch->kv_lens[r] < 1 ||
            (batch->kv_lens[r] + batch->page_size - 1) / batch->page_size > batch->max_pages_per_req)
            return PAT_ERR_BAD_KV_LEN;
    try {
        Entry key;
        std::memset(&key.opts, 0, sizeof key.opts);
        key.opts.force_tile = -1;
        if (opts) key.opts = *opts;
        flatten(*batch, key);
        // 1: the same batch (fingerprint, then every word compared)
        for (auto it = cache->entries.begin(); it != cache->entries.end(); ++it) {
            if (it->fingerprint != key.fingerprint || !same_shape(*it, key) || it->kv_lens != key.kv_lens ||
                it->pages != key.pages)
                continue;
            cache->entries.splice(cache->entries.begin(), cache->entries, it);
            *out_plan = cache->entries.front().plan;
            if (how) *how = 1;
            return PAT_OK;
        }
        // 2: a cached batch some decode steps later: the lazy update in place
        for (auto it = cache->entries.begin(); it != cache->entries.end(); ++it) {
            if (!is_successor(*it, key)) continue;
            const int rc = pat_plan_advance(it->plan, batch->kv_lens, batch->block_tables, batch->max_pages_per_req);
            if (rc != PAT_OK) continue;                   // stale or refused: plan anew below
            key.plan = it->plan;
            *it = std::move(key);
            cache->entries.splice(cache->entries.begin(), cache->entries, it);
            *out_plan = cache->entries.front().plan;
            if (how) *how = 2;
            return PAT_OK;
        }
        // 0: plan anew; the least recently used plan goes when the cache is full
        pat_plan_t *plan = nullptr;
        const int rc = pat_plan(batch, opts, &plan);
        if (rc != PAT_OK) return rc;
        key.plan = plan;
        if (cache->entries.size() >= cache->capacity) {
            pat_plan_destroy(cache->entries.back().plan);
            cache->entries.pop_back();
        }
        try {
            cache->entries.push_front(std::move(key));
        } catch (const std::bad_alloc &) {
            pat_plan_destroy(plan);
            throw;
        }
        *out_plan = plan;
        if (how) *how = 0;
        return PAT_OK;
    } catch (const std::bad_alloc &) {
        return PAT_ERR_OUT_OF_MEMORY;
    }
}

}  // extern "C"
