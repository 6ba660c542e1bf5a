// Host-only driver for the sanitizer build of the planner (AddressSanitizer + UBSan, CPU):
// reads one case written by tests/test_sanitizers.py, plans it, walks every array of the schedule
// and of the device image, then replays the recorded decode steps through the lazy update.
// Exit status 0 = the planner returned what the case expects and no sanitizer report was raised.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pat_internal.h"

namespace pat {
int build_plan(const pat_batch_desc &b, const pat_plan_opts &o, pat_plan_s &pl);
int advance_plan(pat_plan_s &pl, const int32_t *new_kv_lens, const int32_t *block_tables, int32_t W);
void refresh_view(pat_plan_s &pl);
}  // namespace pat

static long long walk(const pat_plan_s &pl)
{
    long long sum = 0;
    auto add = [&](const std::vector<int32_t> &v) { for (int32_t x : v) sum += x; };
    add(pl.item_req_off); add(pl.item_req_ids); add(pl.item_req_slot); add(pl.item_page_off);
    add(pl.item_page_ids); add(pl.item_page_start); add(pl.item_kv_len); add(pl.req_slot_off);
    add(pl.req_slot_ids); add(pl.entry_item); add(pl.entry_row_begin); add(pl.entry_num_rows);
    add(pl.entry_tile); add(pl.entry_heads_per_wg); add(pl.pool_ids); add(pl.item_pool_base);
    add(pl.item_pool_cap); add(pl.item_num_pages); add(pl.item_unit_off); add(pl.item_units);
    add(pl.item_wave_off); add(pl.item_waves); add(pl.kv_lens); add(pl.req_tail_item); add(pl.merge_req);
    for (unsigned char c : pl.staging) sum += c;
    // what the kernels would follow: every id a unit or item names must be inside its array
    const int32_t n_pool = (int32_t)pl.pool_ids.size(), n_req = (int32_t)pl.item_req_ids.size();
    for (const pat::DevUnit &u : pl.units) {
        if (u.e.page_off < 0 || u.e.page_off + u.e.n_pages > n_pool) return -1;
        if (u.e.req_off < 0 || u.e.req_off + u.e.n_req > n_req) return -1;
        if (u.kvh0 < 0 || u.kvh0 + u.n_heads > pl.Hkv || u.e.n_rows < 1) return -1;
        sum += pl.pool_ids[u.e.page_off + u.e.n_pages - 1] + pl.item_req_ids[u.e.req_off + u.e.n_req - 1];
    }
    for (const pat::DevWaveItem &w : pl.wave_items) {
        if (w.page_off < 0 || w.page_off + w.n_pages > n_pool || w.kvh < 0 || w.kvh >= pl.Hkv) return -1;
        if (w.req_off < 0 || w.req_off + w.n_req > n_req) return -1;
        sum += pl.pool_ids[w.page_off + w.n_pages - 1];
    }
    for (const pat::DevWorker &w : pl.workers) {
        if (w.unit_begin < 0 || w.unit_end > (int32_t)pl.units.size() || w.unit_begin > w.unit_end) return -1;
        for (int v = 0; v < 8; ++v)
            if (w.item_off[v] < 0 || w.item_off[v] > w.item_off[v + 1] ||
                w.item_off[v + 1] > (int32_t)pl.wave_items.size())
                return -1;
    }
    return sum < 0 ? -sum : sum;
}

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    FILE *f = std::fopen(argv[1], "rb");
    if (!f) return 2;
    std::vector<int32_t> in;
    int32_t buf[4096];
    size_t n;
    while ((n = std::fread(buf, 4, 4096, f)) > 0) in.insert(in.end(), buf, buf + n);
    std::fclose(f);
    size_t at = 0;
    auto take = [&](size_t k) { const int32_t *p = in.data() + at; at += k; if (at > in.size()) std::exit(2); return p; };
    const int32_t *h = take(17);
    pat_batch_desc b;
    std::memset(&b, 0, sizeof b);
    b.num_requests = h[0]; b.max_pages_per_req = h[1]; b.page_size = h[2]; b.num_pages = h[3];
    b.num_q_heads = h[4]; b.num_kv_heads = h[5]; b.head_dim = 128; b.dtype = h[6];
    pat_plan_opts o;
    std::memset(&o, 0, sizeof o);
    o.mode = h[7]; o.split_policy = h[8]; o.split_target_tokens = h[9]; o.force_tile = h[10];
    o.num_cus = h[11]; o.wave_kv_tokens = h[12]; o.dual_launch = h[13]; o.merge_factor = h[14];
    const int32_t n_adv = h[15], want_rc = h[16];
    const size_t B = (size_t)(h[0] > 0 ? h[0] : 0), W = (size_t)(h[1] > 0 ? h[1] : 0);
    b.block_tables = take(B * W);
    b.kv_lens = take(B);
    pat_plan_s pl;
    int rc = pat::build_plan(b, o, pl);
    if (rc != want_rc) { std::fprintf(stderr, "build_plan rc %d, expected %d\n", rc, want_rc); return 1; }
    if (rc != PAT_OK) return 0;
    long long s = walk(pl);
    if (s < 0) { std::fprintf(stderr, "schedule names an id outside its array\n"); return 1; }
    for (int32_t k = 0; k < n_adv; ++k) {
        const int32_t W2 = *take(1), want = *take(1);
        const int32_t *bt2 = take(B * (size_t)W2);
        const int32_t *kv2 = take(B);
        rc = pat::advance_plan(pl, kv2, bt2, W2);
        if (rc != want) { std::fprintf(stderr, "advance %d rc %d, expected %d\n", k, rc, want); return 1; }
        pat::refresh_view(pl);
        if (walk(pl) < 0) { std::fprintf(stderr, "schedule broken after advance %d\n", k); return 1; }
    }
    std::printf("ok %lld items=%d units=%zu wave_items=%zu\n", s, pl.stats.num_items, pl.units.size(),
                pl.wave_items.size());
    return 0;
}
