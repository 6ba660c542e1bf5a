// Host-only driver for the sanitizer build of the plan cache (AddressSanitizer + UBSan + leak check,
// CPU).  The cache calls the library's pat_plan / pat_plan_advance / pat_plan_destroy, which live in
// the HIP translation unit; here they are stand-ins over the planner's own functions, so that the
// cache and the planner can be built without a GPU compiler.  A fixed scenario: hits, successors
// after decode steps, eviction when full, refused input.  Exit status 0 = every answer as expected.
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "pat_internal.h"

namespace pat {
int build_plan(const pat_batch_desc &b, const pat_plan_opts &o, pat_plan_s &pl);
int advance_plan(pat_plan_s &pl, const int32_t *new_kv_lens, const int32_t *block_tables, int32_t W);
}  // namespace pat

extern "C" {
int pat_plan(const pat_batch_desc *batch, const pat_plan_opts *opts, pat_plan_t **out_plan)
{
    pat_plan_opts o;
    std::memset(&o, 0, sizeof o);
    o.force_tile = -1;
    if (opts) o = *opts;
    pat_plan_s *pl = new (std::nothrow) pat_plan_s();
    if (!pl) return PAT_ERR_OUT_OF_MEMORY;
    const int rc = pat::build_plan(*batch, o, *pl);
    if (rc != PAT_OK) { delete pl; return rc; }
    *out_plan = pl;
    return PAT_OK;
}
int pat_plan_advance(pat_plan_t *plan, const int32_t *kv, const int32_t *bt, int32_t W)
{
    return pat::advance_plan(*plan, kv, bt, W);
}
void pat_plan_destroy(pat_plan_t *plan) { delete plan; }
}

namespace {

struct Batch {
    int32_t B, W;
    std::vector<int32_t> bt, kv;
    pat_batch_desc desc() const
    {
        pat_batch_desc d;
        std::memset(&d, 0x5a, sizeof d);                // padding bytes are the caller's: anything
        d.num_requests = B; d.max_pages_per_req = W; d.block_tables = bt.data(); d.kv_lens = kv.data();
        d.page_size = 16; d.num_pages = 4096; d.num_q_heads = 8; d.num_kv_heads = 2; d.head_dim = 128;
        d.dtype = PAT_BF16; d.num_nodes = 0; d.node_parent = nullptr; d.node_num_pages = nullptr;
        d.req_leaf_node = nullptr;
        return d;
    }
};

// B requests under one shared prefix of `shared` pages, request r with own[r] tokens of its own
Batch make(int32_t B, int32_t shared, int32_t first_page, const std::vector<int32_t> &own, int32_t W)
{
    Batch b{B, W, std::vector<int32_t>((size_t)B * W, 0), std::vector<int32_t>(B)};
    for (int32_t r = 0; r < B; ++r) {
        for (int32_t i = 0; i < shared; ++i) b.bt[(size_t)r * W + i] = first_page + i;
        const int32_t pages = (own[r] + 15) / 16;       // a request's own pages: eight ids kept for it
        for (int32_t i = 0; i < pages; ++i) b.bt[(size_t)r * W + shared + i] = first_page + shared + 8 * r + i;
        b.kv[r] = shared * 16 + own[r];
    }
    return b;
}

int fail(const char *what) { std::fprintf(stderr, "cache driver: %s\n", what); return 1; }

}  // namespace

int main()
{
    pat_plan_cache_t *c = nullptr;
    if (pat_plan_cache_create(0, &c) != PAT_ERR_INVALID_ARG) return fail("capacity 0 accepted");
    if (pat_plan_cache_create(2, &c) != PAT_OK) return fail("create");
    Batch a = make(6, 4, 100, {5, 17, 30, 16, 1, 40}, 12);
    Batch b2 = make(3, 2, 900, {20, 20, 9}, 12);
    Batch c3 = make(4, 1, 1500, {3, 70, 33, 12}, 12);
    pat_plan_t *p = nullptr, *q = nullptr;
    int32_t how = -1;
    pat_batch_desc d = a.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &p, &how) != PAT_OK || how != 0) return fail("first get");
    d = a.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 1 || q != p) return fail("hit");
    // a wider table with the same used entries is the same batch
    Batch wide = make(6, 4, 100, {5, 17, 30, 16, 1, 40}, 20);
    d = wide.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 1 || q != p) return fail("wider table");
    // three decode steps later (one request crosses a page): brought up to date in place
    Batch later = make(6, 4, 100, {8, 20, 33, 19, 4, 43}, 12);
    d = later.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 2 || q != p) return fail("successor");
    if (q->kv_lens[2] != 4 * 16 + 33) return fail("successor not advanced");
    // the old state is gone from the cache: planned anew, which fills the cache (capacity 2)
    d = a.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 0 || q == p) return fail("old state");
    d = b2.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 0) return fail("third batch");
    // `later` was the least recently used: evicted, its plan freed (the leak check sees a miss)
    d = later.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how == 1) return fail("evicted entry hit");
    // other options are another key
    pat_plan_opts o;
    std::memset(&o, 0, sizeof o);
    o.force_tile = -1;
    o.split_policy = PAT_SPLIT_NONE;
    d = later.desc();
    if (pat_plan_cache_get(c, &d, &o, &q, &how) != PAT_OK || how != 0) return fail("options ignored");
    // refused input leaves the cache as it is
    Batch bad = c3;
    bad.kv[1] = 0;
    d = bad.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_ERR_BAD_KV_LEN) return fail("kv_len 0 accepted");
    bad = c3;
    bad.bt[1] = 99999;
    d = bad.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_ERR_BAD_PAGE_ID) return fail("bad page accepted");
    d = c3.desc();
    if (pat_plan_cache_get(c, &d, nullptr, &q, &how) != PAT_OK || how != 0) return fail("fourth batch");
    if (pat_plan_cache_get(nullptr, &d, nullptr, &q, &how) != PAT_ERR_INVALID_ARG) return fail("null cache");
    pat_plan_cache_destroy(c);
    pat_plan_cache_destroy(nullptr);
    std::printf("ok\n");
    return 0;
}
