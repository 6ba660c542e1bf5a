// Pack stage (CPU, integers only): block table -> prefix forest -> TreeHeuristic -> long-KV
// split -> tile selection -> launch schedule.
//
// Follows sec. "Pack Scheduler" (tree-structured block table, inter-node profit rule,
// Algorithm 1 "TreeHeuristic"), sec. "Multi-tile Kernel" (tile selector: round-up rule for m)
// and sec. "Multi Kernel Forward" (long-KV split).  Readings of points the paper leaves open:
//   * the length tested in Algorithm 1 is the token length of the blocks handed to the current
//     call (the node's own run plus every ancestor run merged into it); ties merge;
//   * only pages a request fills completely can be shared;
//   * packs without queries or pages are dropped.
#include <algorithm>
#include <climits>
#include <cstring>
#include <new>
#include <numeric>
#include <queue>

#include "pat_internal.h"

namespace pat {

static const TileInfo kTiles[NUM_TILES] = {
    {16, 4, true},      // TILE_VALU16
    {16, 128, true},    // TILE_STREAM16
    {16, 32, true},     // TILE_WAVE16
    {64, 64, true},     // TILE_PACKED64
    {128, 64, true},    // TILE_PACKED128
};

static bool g_tile_available[NUM_TILES] = {true, true, true, true, true};

const TileInfo &tile_info(int id) { return kTiles[id]; }

void set_tile_available(int id, bool on) { g_tile_available[id] = on; }
bool tile_available(int id) { return id >= 0 && id < NUM_TILES && g_tile_available[id]; }

namespace {

inline bool is_packed_tile(int32_t t) { return t >= TILE_PACKED64; }

struct Node {
    int32_t parent = -1;
    int32_t start = 0;        // first page index in the rows of its requests
    int32_t n_pages = 0;      // pages owned by this node
    int32_t req_begin = 0;    // requests under the node: order[req_begin .. req_end)
    int32_t req_end = 0;
    int32_t first_child = -1, next_sibling = -1, last_child = -1;
    bool leaf = false;
    int32_t size() const { return req_end - req_begin; }
};

struct Pack {
    int32_t start, n_pages, kv_len;
    std::vector<int32_t> reqs;        // ascending
};

struct Forest {
    std::vector<Node> nodes;
    std::vector<int32_t> order;       // requests grouped so every node owns a contiguous range
    std::vector<int32_t> roots;
};

inline int32_t pages_of(int32_t kv_len, int32_t P) { return (kv_len + P - 1) / P; }

void add_child(std::vector<Node> &nodes, int32_t parent, int32_t child)
{
    nodes[child].parent = parent;
    if (parent < 0) return;
    if (nodes[parent].first_child < 0)
        nodes[parent].first_child = child;
    else
        nodes[nodes[parent].last_child].next_sibling = child;
    nodes[parent].last_child = child;
}

// Derive the forest from identical leading page ids.  Requests are kept in a permutation
// array; each recursion level regroups a sub-range by the page id at the current depth, so
// every (request, page) is looked at a constant number of times.
void derive_forest(const pat_batch_desc &b, Forest &f)
{
    const int32_t B = b.num_requests, P = b.page_size, W = b.max_pages_per_req;
    f.order.resize(B);
    std::iota(f.order.begin(), f.order.end(), 0);
    struct Work { int32_t begin, end, depth, parent; };
    std::vector<Work> stack;
    stack.push_back({0, B, 0, -1});
    auto row = [&](int32_t r) { return b.block_tables + (int64_t)r * W; };
    auto full = [&](int32_t r) { return b.kv_lens[r] / P; };
    std::vector<std::pair<int64_t, int32_t>> keyed;
    while (!stack.empty()) {
        Work w = stack.back();
        stack.pop_back();
        // key = page id at this depth for requests that can still share, else unique negative
        keyed.clear();
        for (int32_t i = w.begin; i < w.end; ++i) {
            int32_t r = f.order[i];
            int64_t key = w.depth < full(r) ? (int64_t)row(r)[w.depth] : -(int64_t)r - 1;
            keyed.push_back({key, r});
        }
        // group equal keys; keep groups in order of their smallest request id
        std::stable_sort(keyed.begin(), keyed.end(),
                         [](const auto &a, const auto &c) { return a.first < c.first; });
        struct Grp { int32_t lo, hi, min_req; };
        std::vector<Grp> groups;
        for (size_t i = 0; i < keyed.size();) {
            size_t j = i;
            int32_t mn = keyed[i].second;
            while (j < keyed.size() && keyed[j].first == keyed[i].first) {
                mn = std::min(mn, keyed[j].second);
                ++j;
            }
            groups.push_back({(int32_t)i, (int32_t)j, mn});
            i = j;
        }
        std::sort(groups.begin(), groups.end(),
                  [](const Grp &a, const Grp &c) { return a.min_req < c.min_req; });
        int32_t pos = w.begin;
        std::vector<Work> pending;
        for (const Grp &g : groups) {
            int32_t lo = pos;
            for (int32_t i = g.lo; i < g.hi; ++i) f.order[pos++] = keyed[i].second;
            std::sort(f.order.begin() + lo, f.order.begin() + pos);
            Node n;
            n.start = w.depth;
            n.req_begin = lo;
            n.req_end = pos;
            if (pos - lo == 1) {
                int32_t r = f.order[lo];
                n.leaf = true;
                n.n_pages = pages_of(b.kv_lens[r], P) - w.depth;
            } else {
                // longest run of identical, completely filled pages shared by the group
                int32_t r0 = f.order[lo];
                int32_t run = full(r0) - w.depth;
                for (int32_t i = lo + 1; i < pos && run > 0; ++i) {
                    int32_t r = f.order[i];
                    run = std::min(run, full(r) - w.depth);
                    const int32_t *a = row(r0) + w.depth, *c = row(r) + w.depth;
                    int32_t k = 0;
                    while (k < run && a[k] == c[k]) ++k;
                    run = k;
                }
                n.n_pages = run;      // >= 1 because the group agreed on the page at depth
            }
            f.nodes.push_back(n);
            int32_t id = (int32_t)f.nodes.size() - 1;
            add_child(f.nodes, w.parent, id);
            if (w.parent < 0) f.roots.push_back(id);
            if (!n.leaf) pending.push_back({lo, pos, w.depth + n.n_pages, id});
        }
        // depth-first, children of earlier groups first: push in reverse
        for (auto it = pending.rbegin(); it != pending.rend(); ++it) stack.push_back(*it);
    }
}

// Build the forest from the caller's explicit tree and check it against the block tables.
int explicit_forest(const pat_batch_desc &b, Forest &f)
{
    const int32_t B = b.num_requests, P = b.page_size, W = b.max_pages_per_req, N = b.num_nodes;
    if (!b.node_parent || !b.node_num_pages || !b.req_leaf_node) return PAT_ERR_INVALID_ARG;
    std::vector<int32_t> start(N, 0), count(N, 0);
    for (int32_t i = 0; i < N; ++i) {
        int32_t p = b.node_parent[i];
        if (p >= i || p < -1 || b.node_num_pages[i] < 0) return PAT_ERR_BAD_TREE;
        start[i] = p < 0 ? 0 : start[p] + b.node_num_pages[p];
    }
    // requests per node (every ancestor of the leaf node)
    std::vector<std::vector<int32_t>> members(N);
    for (int32_t r = 0; r < B; ++r) {
        int32_t leaf = b.req_leaf_node[r];
        if (leaf < 0 || leaf >= N) return PAT_ERR_BAD_TREE;
        if (start[leaf] + b.node_num_pages[leaf] != pages_of(b.kv_lens[r], P))
            return PAT_ERR_BAD_TREE;
        for (int32_t u = leaf; u >= 0; u = b.node_parent[u]) members[u].push_back(r);
    }
    for (int32_t i = 0; i < N; ++i) {
        if (members[i].size() < 2) continue;
        int32_t r0 = members[i][0];
        for (int32_t r : members[i]) {
            if (b.kv_lens[r] / P < start[i] + b.node_num_pages[i]) return PAT_ERR_BAD_TREE;
            if (std::memcmp(b.block_tables + (int64_t)r * W + start[i],
                            b.block_tables + (int64_t)r0 * W + start[i],
                            sizeof(int32_t) * (size_t)b.node_num_pages[i]) != 0)
                return PAT_ERR_BAD_TREE;
        }
    }
    // Walk the caller's tree depth-first so that every node owns a contiguous range of the
    // request permutation.  A node with a single request below it becomes that request's
    // leaf (with everything beneath it).  Requests that end in a shared node get an empty
    // leaf under it, so that "one leaf per request" holds as in the derived forest.
    std::vector<std::vector<int32_t>> kids(N), ends_here(N);
    for (int32_t i = 0; i < N; ++i)
        if (b.node_parent[i] >= 0) kids[b.node_parent[i]].push_back(i);
    for (int32_t r = 0; r < B; ++r) ends_here[b.req_leaf_node[r]].push_back(r);
    f.order.clear();
    f.nodes.clear();
    struct Visit { int32_t node, parent_out, out_id; bool close; };
    std::vector<Visit> st;
    for (int32_t i = N - 1; i >= 0; --i)
        if (b.node_parent[i] < 0 && !members[i].empty()) st.push_back({i, -1, -1, false});
    while (!st.empty()) {
        Visit cur = st.back();
        st.pop_back();
        const int32_t u = cur.node;
        if (cur.close) {
            f.nodes[cur.out_id].req_end = (int32_t)f.order.size();
            continue;
        }
        Node n;
        n.start = start[u];
        n.req_begin = (int32_t)f.order.size();
        if (members[u].size() == 1) {
            int32_t r = members[u][0];
            n.leaf = true;
            n.n_pages = pages_of(b.kv_lens[r], P) - start[u];
            f.order.push_back(r);
            n.req_end = (int32_t)f.order.size();
            f.nodes.push_back(n);
            int32_t id = (int32_t)f.nodes.size() - 1;
            add_child(f.nodes, cur.parent_out, id);
            if (cur.parent_out < 0) f.roots.push_back(id);
            continue;
        }
        n.n_pages = b.node_num_pages[u];
        f.nodes.push_back(n);
        const int32_t id = (int32_t)f.nodes.size() - 1;
        add_child(f.nodes, cur.parent_out, id);
        if (cur.parent_out < 0) f.roots.push_back(id);
        for (int32_t r : ends_here[u]) {
            Node l;
            l.leaf = true;
            l.start = start[u] + b.node_num_pages[u];
            l.n_pages = 0;
            l.req_begin = (int32_t)f.order.size();
            f.order.push_back(r);
            l.req_end = (int32_t)f.order.size();
            f.nodes.push_back(l);
            add_child(f.nodes, id, (int32_t)f.nodes.size() - 1);
        }
        st.push_back({u, cur.parent_out, id, true});
        for (auto it = kids[u].rbegin(); it != kids[u].rend(); ++it)
            if (!members[*it].empty()) st.push_back({*it, id, -1, false});
    }
    if ((int32_t)f.order.size() != B) return PAT_ERR_BAD_TREE;
    for (Node &n : f.nodes)
        std::sort(f.order.begin() + n.req_begin, f.order.begin() + n.req_end);
    return PAT_OK;
}

struct Packer {
    const pat_batch_desc &b;
    const Forest &f;
    int32_t merge_factor;
    std::vector<Pack> packs;
    int32_t merged_children = 0;

    void emit(const int32_t *reqs, int32_t n, int32_t start, int32_t n_pages)
    {
        if (n == 0 || n_pages == 0) return;
        Pack p;
        p.start = start;
        p.n_pages = n_pages;
        p.reqs.assign(reqs, reqs + n);
        std::sort(p.reqs.begin(), p.reqs.end());
        if (n == 1)
            p.kv_len = std::min(b.kv_lens[reqs[0]], (start + n_pages) * b.page_size) -
                       start * b.page_size;
        else
            p.kv_len = n_pages * b.page_size;
        packs.push_back(std::move(p));
    }

    // Algorithm 1 with an explicit stack.  A frame carries the blocks handed to the call as
    // the contiguous page range [start, start + n_pages) of the node's requests' rows.
    void tree_heuristic(int32_t root)
    {
        struct Frame { int32_t node, start, n_pages; };
        std::vector<Frame> stack;
        stack.push_back({root, f.nodes[root].start, f.nodes[root].n_pages});
        std::vector<int32_t> remaining;
        std::vector<char> taken(b.num_requests, 0);
        while (!stack.empty()) {
            Frame fr = stack.back();
            stack.pop_back();
            const Node &n = f.nodes[fr.node];
            if (n.leaf) {
                emit(&f.order[n.req_begin], 1, fr.start, fr.n_pages);
                continue;
            }
            const int64_t blocks_len = (int64_t)fr.n_pages * b.page_size;
            for (int32_t c = n.first_child; c >= 0; c = f.nodes[c].next_sibling) {
                const Node &cn = f.nodes[c];
                if ((int64_t)merge_factor * cn.size() < blocks_len) {
                    stack.push_back({c, cn.start, cn.n_pages});               // Scheme 1
                } else {
                    stack.push_back({c, fr.start, fr.n_pages + cn.n_pages});  // Scheme 2
                    for (int32_t i = cn.req_begin; i < cn.req_end; ++i) taken[f.order[i]] = 1;
                    ++merged_children;
                }
            }
            remaining.clear();
            for (int32_t i = n.req_begin; i < n.req_end; ++i) {
                int32_t r = f.order[i];
                if (!taken[r]) remaining.push_back(r);
                taken[r] = 0;     // a request is taken at most once per level of the walk
            }
            emit(remaining.data(), (int32_t)remaining.size(), fr.start, fr.n_pages);
        }
    }

    void per_node(int32_t root)
    {
        std::vector<int32_t> stack{root};
        while (!stack.empty()) {
            int32_t u = stack.back();
            stack.pop_back();
            const Node &n = f.nodes[u];
            emit(&f.order[n.req_begin], n.size(), n.start, n.n_pages);
            for (int32_t c = n.first_child; c >= 0; c = f.nodes[c].next_sibling)
                stack.push_back(c);
        }
    }
};

int validate(const pat_batch_desc &b)
{
    if (b.num_requests < 1 || b.max_pages_per_req < 1 || !b.block_tables || !b.kv_lens)
        return PAT_ERR_INVALID_ARG;
    if (b.num_q_heads < 1 || b.num_kv_heads < 1 || b.num_q_heads % b.num_kv_heads != 0)
        return PAT_ERR_INVALID_ARG;
    if (b.num_pages < 1) return PAT_ERR_INVALID_ARG;
    if (b.head_dim != 128 || b.page_size != 16) return PAT_ERR_UNSUPPORTED;
    if (b.dtype != PAT_F16 && b.dtype != PAT_BF16) return PAT_ERR_UNSUPPORTED;
    for (int32_t r = 0; r < b.num_requests; ++r) {
        int32_t n = b.kv_lens[r];
        if (n < 1 || pages_of(n, b.page_size) > b.max_pages_per_req) return PAT_ERR_BAD_KV_LEN;
        const int32_t *row = b.block_tables + (int64_t)r * b.max_pages_per_req;
        for (int32_t i = 0, np = pages_of(n, b.page_size); i < np; ++i)
            if (row[i] < 0 || row[i] >= b.num_pages) return PAT_ERR_BAD_PAGE_ID;
    }
    return PAT_OK;
}

// Tile selector (sec. "Multi-tile Kernel", "Tile Selection": m from the number of query rows, n
// from the KV length).
//   m: the smallest available m that holds the rows; above the largest m the caller cuts the rows
//      into equal blocks.  For 17..32 rows a short node is cheaper as two 16-row blocks than as one
//      64-row packed workgroup (start-up and epilogue of the packed tile outweigh reading the
//      node twice through L2): the crossover, measured with the KV-length sweep of the
//      calibration module, is kPackedMinTokens.
//   n: the 16-row family has two KV tiles: n = 32 (TILE_WAVE16, one wavefront per item) for
//      entries of up to `wave_kv` tokens where the launch runs many rounds (wave_kv = 0: never),
//      n = 128 (TILE_STREAM16, four wavefronts per KV head) otherwise.
constexpr int32_t kPackedMinTokens = 48;
int32_t select_tile(int32_t rows, int32_t kv_len, int32_t wave_kv, int32_t packed_min)
{
    if (rows <= 16 || (rows <= 32 && kv_len < packed_min)) {
        if (wave_kv > 0 && kv_len <= wave_kv && g_tile_available[TILE_WAVE16]) return TILE_WAVE16;
        if (g_tile_available[TILE_STREAM16]) return TILE_STREAM16;
    }
    int32_t best = -1;
    for (int32_t t = 0; t < NUM_TILES; ++t) {
        if (!g_tile_available[t] || !is_packed_tile(t)) continue;
        if (kTiles[t].m >= rows && (best < 0 || kTiles[t].m < kTiles[best].m)) best = t;
    }
    if (best >= 0) return best;
    // no packed tile holds the rows: the largest available one, else a 16-row tile
    for (int32_t t = NUM_TILES - 1; t >= 0; --t)
        if (g_tile_available[t] && is_packed_tile(t)) return t;
    return g_tile_available[TILE_STREAM16] ? TILE_STREAM16 : TILE_VALU16;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

int build_plan(const pat_batch_desc &b, const pat_plan_opts &o, pat_plan_s &pl)
{
    int rc = validate(b);
    if (rc != PAT_OK) return rc;
    if (o.mode < PAT_MODE_PAT || o.mode > PAT_MODE_NO_SHARING) return PAT_ERR_INVALID_ARG;
    if (o.split_policy < PAT_SPLIT_AUTO || o.split_policy > PAT_SPLIT_TARGET)
        return PAT_ERR_INVALID_ARG;
    if (o.split_policy == PAT_SPLIT_TARGET && o.split_target_tokens < 1)
        return PAT_ERR_INVALID_ARG;
    if (o.merge_factor < 0 || o.num_cus < 0 || o.packed_min_tokens < 0) return PAT_ERR_INVALID_ARG;
    if (o.fused_merge < -1 || o.fused_merge > 1 || o.dual_launch < -1 || o.dual_launch > 1) return PAT_ERR_INVALID_ARG;
    if (o.force_tile < -1 || o.force_tile >= NUM_TILES) return PAT_ERR_INVALID_ARG;
    if (o.force_tile >= 0 && !g_tile_available[o.force_tile]) return PAT_ERR_UNSUPPORTED;
    for (int32_t x : o.reserved)
        if (x != 0) return PAT_ERR_INVALID_ARG;
    for (int32_t x : o.model_ns)
        if (x < 0) return PAT_ERR_INVALID_ARG;
    if ((o.model_ns[0] || o.model_ns[1] || o.model_ns[2] || o.model_ns[3]) &&
        (o.model_ns[1] < 1 || o.model_ns[3] < 1))
        return PAT_ERR_INVALID_ARG;                       // per-token costs must be positive

    const int32_t B = b.num_requests, P = b.page_size, W = b.max_pages_per_req;
    const int32_t G = b.num_q_heads / b.num_kv_heads;
    pl.B = B; pl.Hq = b.num_q_heads; pl.Hkv = b.num_kv_heads; pl.d = b.head_dim; pl.P = P;
    pl.dtype = b.dtype; pl.num_pages = b.num_pages; pl.opts = o;

    // ---- forest ----------------------------------------------------------------------
    Forest f;
    if (o.mode == PAT_MODE_NO_SHARING) {
        f.order.resize(B);
        std::iota(f.order.begin(), f.order.end(), 0);
        for (int32_t r = 0; r < B; ++r) {
            Node n;
            n.leaf = true; n.start = 0; n.n_pages = pages_of(b.kv_lens[r], P);
            n.req_begin = r; n.req_end = r + 1;
            f.nodes.push_back(n);
            f.roots.push_back(r);
        }
    } else if (b.num_nodes > 0) {
        rc = explicit_forest(b, f);
        if (rc != PAT_OK) return rc;
    } else {
        derive_forest(b, f);
    }

    // ---- packs -----------------------------------------------------------------------
    Packer pk{b, f, o.merge_factor > 0 ? o.merge_factor : 4, {}, 0};
    for (int32_t root : f.roots) {
        if (o.mode == PAT_MODE_PAT) pk.tree_heuristic(root);
        else pk.per_node(root);
    }
    std::vector<Pack> &packs = pk.packs;
    int64_t unique_tokens = 0;
    for (const Pack &p : packs) unique_tokens += p.kv_len;

    // ---- long-KV split -----------------------------------------------------------------
    struct Item { int32_t pack, start, n_pages, kv_len, heads_per_wg; bool wave; };
    std::vector<Item> items;
    // Run-time model (ns) of the device-aware split and of the static schedule of launches with
    // wavefront items, measured on MI355X with every CU busy (L = tokens, h = KV heads):
    //   packed workgroup : 13000 + 26 L     (first tile late, tiles computed in turn, many
    //                                        partial rows to write); 64-row tile: 0.73 and 0.90 of it
    //   16-row workgroup :  4000 + 20 h L   (its share of the HBM stream)
    //   wavefront item   :  1500 + 160 L    (an eighth of a CU's stream; start-up hidden)
    const bool own_model = o.model_ns[0] || o.model_ns[1] || o.model_ns[2] || o.model_ns[3];
    const int64_t c0p = own_model ? o.model_ns[0] : 13000, c1p = own_model ? o.model_ns[1] : 26;
    const int64_t c0q = c0p * 73 / 100, c1q = std::max<int64_t>(1, c1p * 90 / 100);
    const int64_t c0s = own_model ? o.model_ns[2] : 4000, c1s = own_model ? o.model_ns[3] : 20;
    const int64_t c0w = 1500, c1w = 8 * c1s;
    const int32_t packed_min = o.packed_min_tokens > 0 ? o.packed_min_tokens : kPackedMinTokens;
    // Two-kernel launch: 16-row tiles as 256-thread workgroups of one KV head, two per CU.
    const bool dual = o.dual_launch > 0 && o.force_tile != TILE_WAVE16 && !(o.wave_kv_tokens > 0);
    // TILE_WAVE16 (n = 32, one wavefront per item): where 16-row packs of a launch of many rounds
    // are short.  wave_kv = longest item, wave_max = longest pack that is cut into such items.
    int32_t wave_kv = 0, wave_max = 0;
    if (o.force_tile == TILE_WAVE16) {
        wave_kv = wave_max = INT32_MAX;
    } else if (o.force_tile < 0 && o.wave_kv_tokens >= 0 && g_tile_available[TILE_WAVE16]) {
        const bool many_rounds = (unique_tokens * b.num_kv_heads + (o.num_cus > 0 ? o.num_cus : 256) - 1) /
                                 (o.num_cus > 0 ? o.num_cus : 256) > 1024;
        // Measured on MI355X (the calibration module's KV-length sweep, C3, C4): on a batch of
        // nothing but short unshared requests the n = 32 tile beats the n = 128 tile up to about
        // 384 tokens (by 36 % at 64 tokens, 21 % at 128, 7 % at 256); next to packed tiles or long
        // streams it does not (C3, C4: equal to 20 % slower -- eight independent streams per CU
        // crowd the packed tiles' loads out, and the static lists start behind the units).  So the
        // planner picks it for launches of many rounds in which EVERY pack is such a request.
        // Very short 16-row packs are another matter: a workgroup's start and end cost more than
        // their stream, and as wavefront items they win even beside packed tiles (256 leaves of 64
        // tokens under a 2048-token prefix: 46.8 -> 35.8 us with 32/8 heads, 103.7 -> 67.4 with 32/32;
        // equal at 128 tokens).  Taken where every 16-row pack has at most 96 tokens and they would
        // fill more than one round of workgroups by themselves.
        const bool auto_wave = o.split_policy == PAT_SPLIT_AUTO && o.wave_kv_tokens == 0;
        bool all_short = many_rounds && auto_wave, leaves_short = auto_wave;
        int64_t short_wgs = 0;
        for (size_t i = 0; i < packs.size(); ++i) {
            const int64_t rows = (int64_t)packs[i].reqs.size() * G;
            all_short = all_short && rows <= 16 && packs[i].kv_len <= 384;
            if (rows > 32 || (rows > 16 && packs[i].kv_len >= packed_min)) continue;      // a packed tile
            leaves_short = leaves_short && packs[i].kv_len <= 96;
            short_wgs += (rows + 15) / 16 * ((b.num_kv_heads + 1) / 2);
        }
        leaves_short = leaves_short && short_wgs > (o.num_cus > 0 ? o.num_cus : 256);
        if (o.wave_kv_tokens > 0) {
            wave_kv = o.wave_kv_tokens;
            wave_max = o.wave_max_tokens > 0 ? o.wave_max_tokens : 4 * wave_kv;
        } else if (all_short) {
            wave_kv = wave_max = 384;
        } else if (leaves_short) {
            wave_kv = wave_max = 96;
        }
    }
    {
        // Per pack: into how many parts its KV range is cut, and how many KV heads one
        // workgroup of a 16-row tile serves (2 = one per 256-thread half, 1 = second half idle);
        // wave: the parts run as wavefront items.
        struct Cut { int64_t parts; int32_t heads_per_wg; bool wave = false; };
        std::vector<Cut> cuts(packs.size(), Cut{1, 2});
        auto parts_for = [](const Pack &p, int64_t num, int64_t den) {     // ceil(len / (num/den))
            int64_t parts = 1;
            if ((int64_t)p.kv_len * den > num) parts = ((int64_t)p.kv_len * den + num - 1) / num;
            return std::min<int64_t>(parts, p.n_pages);
        };
        switch (o.split_policy) {
        case PAT_SPLIT_MEAN:
            // (sec. "Multi Kernel Forward", "Long KV Split": parts that keep the length under the
            // mean.)  Parts are whole pages: while the longest part, the first, is still over the
            // mean and has more than one page, cut once more.
            for (size_t i = 0; i < packs.size(); ++i) {
                const int64_t pages = packs[i].n_pages, n = (int64_t)packs.size();
                int64_t parts = parts_for(packs[i], unique_tokens, n);
                while (parts > 1 && parts < pages && (pages + parts - 1) / parts * P * n > unique_tokens) ++parts;
                cuts[i].parts = parts;
            }
            break;
        case PAT_SPLIT_NONE: break;
        case PAT_SPLIT_TARGET:
            for (size_t i = 0; i < packs.size(); ++i)
                cuts[i].parts = parts_for(packs[i], o.split_target_tokens, 1);
            break;
        default: {
            // Device-aware cuts.  One 512-thread workgroup is resident per CU; `slots` of them
            // run at once and share the HBM bandwidth evenly.
            // Small batches run as ONE round: the smallest bound on a workgroup's run time for
            // which the workgroups still fit the slots, so that nothing waits for a second
            // round and all workgroups end together.  Run times follow the model above.
            // A 16-row pack over the bound first goes to one head per workgroup (more CUs, no
            // extra partials), then its KV range is cut.
            // Large batches run many rounds; there two cuts are compared under the same model
            // (see below).
            const int64_t slots = o.num_cus > 0 ? o.num_cus : 256;
            int32_t max_m = 16;
            for (int32_t t = 0; t < NUM_TILES; ++t)
                if (g_tile_available[t]) max_m = std::max(max_m, kTiles[t].m);
            const int64_t Hkv = b.num_kv_heads, pair_wgs = (Hkv + 1) / 2;
            auto packed_c0 = [&](const Pack &p) { return (int64_t)p.reqs.size() * G <= 64 ? c0q : c0p; };
            auto packed_c1 = [&](const Pack &p) { return (int64_t)p.reqs.size() * G <= 64 ? c1q : c1p; };
            auto is_packed = [&](const Pack &p) {
                const int64_t rows = (int64_t)p.reqs.size() * G;
                return rows > 32 || (rows > 16 && p.kv_len >= packed_min);
            };
            auto is_wave = [&](const Pack &p) { return !is_packed(p) && wave_kv > 0 && p.kv_len <= wave_max; };
            // bound = run time in ns a workgroup may take
            auto cut_for = [&](const Pack &p, int64_t bound, bool single_heads) {
                if (is_packed(p))
                    return Cut{parts_for(p, std::max<int64_t>(bound - packed_c0(p), 64 * packed_c1(p)), packed_c1(p)), 1};
                const int64_t room = std::max<int64_t>(bound - c0s, 64 * c1s);
                const int64_t two = parts_for(p, room, 2 * c1s);      // parts with two heads
                if (!single_heads || Hkv < 2) return Cut{two, 2};
                const int64_t one = parts_for(p, room, c1s);          // parts with one head
                // as many workgroups either way: prefer fewer parts (fewer partials to merge)
                return one * Hkv <= two * pair_wgs ? Cut{one, 1} : Cut{two, 2};
            };
            auto workgroups = [&](int64_t bound, bool single_heads) {
                int64_t n = 0;
                for (const Pack &p : packs) {
                    const Cut c = cut_for(p, bound, single_heads);
                    const int64_t rows = (int64_t)p.reqs.size() * G;
                    const int64_t wgs = is_packed(p) ? Hkv : (c.heads_per_wg == 1 ? Hkv : pair_wgs);
                    n += c.parts * (is_packed(p) ? (rows + max_m - 1) / max_m : (rows + 15) / 16) * wgs;
                }
                return n;
            };
            int64_t longest = 0;
            for (const Pack &p : packs)
                longest = std::max<int64_t>(longest, is_packed(p) ? packed_c0(p) + packed_c1(p) * p.kv_len
                                                                : c0s + 2 * c1s * p.kv_len);
            const int64_t share = (unique_tokens * Hkv + slots - 1) / slots;     // token-heads per slot
            // A launch played through with the run-time model: workgroups longest first, a CU takes the
            // next one when it is free (wavefront items as workgroups that hold eight of them side by side).
            auto wg_ns = [&](const Pack &p, const Cut &c) {
                const int64_t L = (p.kv_len + c.parts - 1) / c.parts;
                if (c.wave) return c0w + c1w * L;
                return is_packed(p) ? packed_c0(p) + packed_c1(p) * L : c0s + c.heads_per_wg * c1s * L;
            };
            auto wg_count = [&](const Pack &p, const Cut &c) {
                const int64_t rows = (int64_t)p.reqs.size() * G;
                if (c.wave) return (c.parts * ((rows + 15) / 16) * Hkv + 7) / 8;
                const int64_t wgs = is_packed(p) ? Hkv : (c.heads_per_wg == 1 ? Hkv : pair_wgs);
                return c.parts * (is_packed(p) ? (rows + max_m - 1) / max_m : (rows + 15) / 16) * wgs;
            };
            auto launch_ns = [&](const std::vector<Cut> &cs) {
                std::vector<std::pair<int64_t, int64_t>> jobs;          // (run time, how many)
                for (size_t i = 0; i < packs.size(); ++i)
                    jobs.emplace_back(wg_ns(packs[i], cs[i]), wg_count(packs[i], cs[i]));
                std::sort(jobs.begin(), jobs.end(), std::greater<>());
                std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> busy;
                for (int64_t k = 0; k < slots; ++k) busy.push(0);
                int64_t end = 0;
                for (const auto &j : jobs)
                    for (int64_t k = 0; k < j.second; ++k) {
                        const int64_t t = busy.top() + j.first;
                        busy.pop();
                        busy.push(t);
                        end = std::max(end, t);
                    }
                return end;
            };
            auto many_rounds_cut = [&]() {
                // Workgroups are launched longest first and a CU takes the next one when it is
                // free.  Two candidate cuts are played through that way with the run-time model
                // above; the coarse one is taken unless it ends more than 5 % later (every cut costs
                // one more partial per row to write and merge, which the model does not price):
                //   coarse: only a pack whose workgroup would run clearly longer than the whole
                //           launch is estimated to take is cut, into parts that do not;
                //   fine:   a pack is cut where it exceeds half a slot's share of all
                //           token-heads, whatever its tile.
                std::vector<Cut> fine(packs.size(), Cut{1, 2}), coarse(packs.size(), Cut{1, 2});
                int64_t total_ns = 0;
                for (size_t i = 0; i < packs.size(); ++i) {
                    if (is_wave(packs[i])) {
                        fine[i] = coarse[i] = Cut{parts_for(packs[i], wave_kv, 1), 1, true};
                    } else {
                        fine[i].parts = parts_for(packs[i], (share + 1) / 2, 1);
                    }
                    total_ns += wg_ns(packs[i], coarse[i]) * wg_count(packs[i], coarse[i]);
                }
                const int64_t whole = (total_ns + slots - 1) / slots;         // the launch, if it packed perfectly
                for (size_t i = 0; i < packs.size(); ++i) {
                    const Pack &p = packs[i];
                    if (coarse[i].wave) continue;
                    if (wg_ns(p, coarse[i]) * 100 <= whole * 115) continue;    // (the estimate is no better than that)
                    const int64_t c0 = is_packed(p) ? packed_c0(p) : c0s, c1 = is_packed(p) ? packed_c1(p) : 2 * c1s;
                    coarse[i].parts = parts_for(p, std::max<int64_t>(whole - c0, 64 * c1), c1);
                }
                cuts = launch_ns(coarse) * 100 <= launch_ns(fine) * 105 ? coarse : fine;
            };
            if (share > 1024) {                          // many rounds
                many_rounds_cut();
                break;
            }
            const int64_t floor_bound = std::max(c0p, c0s) + 2000;
            int64_t bound;
            // (two-kernel launches: a 16-row workgroup holds one KV head and half a CU; two of them
            // are counted as one workgroup of two heads)
            const bool single_heads = !dual;
            if (workgroups(floor_bound, single_heads) <= slots) {
                bound = floor_bound;
            } else {
                int64_t lo = floor_bound, hi = std::max(longest, floor_bound + 1);   // W(hi) minimal
                if (workgroups(hi, single_heads) > slots) {
                    // Cannot fit one round anyway: a few rounds.  Bounds on a workgroup's run time
                    // from the floor up to the longest uncut workgroup, a third apart, are each
                    // played through the launch (longest first, a CU takes the next when free); the
                    // coarsest cut within 3 % of the earliest end is taken (every part more is one
                    // more partial per row to write and merge; priced as its bytes, 2 x 516 per q
                    // head, at 4 bytes/ns, on top of the launch).
                    std::vector<Cut> trial(packs.size(), Cut{1, 2}), best;
                    std::vector<std::pair<int64_t, std::vector<Cut>>> played;
                    int64_t earliest = INT64_MAX;
                    for (int64_t t = floor_bound;; t = t * 4 / 3) {
                        const int64_t tb = std::min(t, hi);
                        for (size_t i = 0; i < packs.size(); ++i)
                            trial[i] = is_wave(packs[i]) ? Cut{parts_for(packs[i], wave_kv, 1), 1, true}
                                                         : cut_for(packs[i], tb, false);
                        int64_t partial_rows = 0;
                        for (size_t i = 0; i < packs.size(); ++i)
                            partial_rows += trial[i].parts * (int64_t)packs[i].reqs.size();
                        const int64_t end = launch_ns(trial) + partial_rows * b.num_q_heads * (2 * 516) / 4000;
                        earliest = std::min(earliest, end);
                        played.emplace_back(end, trial);
                        if (tb == hi) break;
                    }
                    for (auto it = played.rbegin(); it != played.rend(); ++it)      // coarsest first
                        if (it->first * 100 <= earliest * 103) { cuts = it->second; break; }
                    break;
                }
                while (lo + 1 < hi) {                               // W(lo) > slots >= W(hi)
                    const int64_t mid = (lo + hi) / 2;
                    if (workgroups(mid, single_heads) <= slots) hi = mid; else lo = mid;
                }
                bound = hi;
            }
            for (size_t i = 0; i < packs.size(); ++i) cuts[i] = cut_for(packs[i], bound, single_heads);
            break;
        }
        }
        if (wave_kv > 0)
            for (size_t i = 0; i < packs.size(); ++i) {
                const Pack &p = packs[i];
                const int64_t rows = (int64_t)p.reqs.size() * G;
                const bool packed = rows > 32 || (rows > 16 && p.kv_len >= packed_min);
                if (cuts[i].wave || o.force_tile == TILE_WAVE16) {
                    cuts[i].wave = true;
                } else if (!packed && p.kv_len <= wave_max && o.wave_kv_tokens > 0) {
                    // an explicit wave_kv_tokens: whatever the policy cut, cut again where needed
                    cuts[i].parts = std::max(cuts[i].parts, parts_for(p, wave_kv, 1));
                    cuts[i].wave = true;
                }
            }
        for (int32_t pi = 0; pi < (int32_t)packs.size(); ++pi) {
            const Pack &p = packs[pi];
            const int64_t parts = cuts[pi].parts;
            int32_t base = p.n_pages / (int32_t)parts, extra = p.n_pages % (int32_t)parts;
            int32_t start = p.start;
            for (int32_t i = 0; i < parts; ++i) {
                int32_t n = base + (i < extra ? 1 : 0);
                int32_t end_tok = (start + n - p.start) * P;
                int32_t tok = std::min(p.kv_len, end_tok) - (start - p.start) * P;
                items.push_back({pi, start, n, tok, cuts[pi].heads_per_wg, cuts[pi].wave});
                start += n;
            }
        }
    }

    // ---- order items: heaviest first (bytes read dominate; rows add compute) -------------
    std::vector<int32_t> perm(items.size());
    std::iota(perm.begin(), perm.end(), 0);
    std::stable_sort(perm.begin(), perm.end(), [&](int32_t a, int32_t c) {
        return items[a].kv_len > items[c].kv_len;
    });

    // ---- per-request partial counts, slots ------------------------------------------------
    std::vector<int32_t> n_parts(B, 0);
    for (const Item &it : items)
        for (int32_t r : packs[it.pack].reqs) ++n_parts[r];
    for (int32_t r = 0; r < B; ++r)
        if (n_parts[r] == 0) return PAT_ERR_INVALID_ARG;     // cannot happen: kv_len >= 1

    const int32_t n_items = (int32_t)items.size();
    pl.item_req_off.assign(1, 0);
    pl.item_page_off.assign(1, 0);
    std::vector<std::vector<int32_t>> req_slots(B);
    std::vector<int32_t> item_heads;
    int32_t n_slots = 0;
    const int32_t tail_reserve =
        o.tail_reserve_pages == 0 ? 16 : std::max<int32_t>(0, o.tail_reserve_pages);
    pl.req_tail_item.assign(B, -1);
    pl.kv_lens.assign(b.kv_lens, b.kv_lens + B);
    for (int32_t k = 0; k < n_items; ++k) {
        const Item &it = items[perm[k]];
        const Pack &p = packs[it.pack];
        for (int32_t r : p.reqs) {
            pl.item_req_ids.push_back(r);
            if (n_parts[r] == 1) {
                pl.item_req_slot.push_back(-1);
            } else {
                pl.item_req_slot.push_back(n_slots);
                req_slots[r].push_back(n_slots);
                ++n_slots;
            }
        }
        const int32_t *row = b.block_tables + (int64_t)p.reqs[0] * W;
        for (int32_t i = 0; i < it.n_pages; ++i) pl.item_page_ids.push_back(row[it.start + i]);
        // device pool: the same ids, and room to grow behind a request's own last item
        pl.item_pool_base.push_back((int32_t)pl.pool_ids.size());
        for (int32_t i = 0; i < it.n_pages; ++i) pl.pool_ids.push_back(row[it.start + i]);
        int32_t cap = it.n_pages;
        if (p.reqs.size() == 1) {
            const int32_t r = p.reqs[0];
            const int32_t req_pages = (b.kv_lens[r] + P - 1) / P;
            if (it.start + it.n_pages == req_pages) {
                pl.req_tail_item[r] = k;
                for (int32_t i = 0; i < tail_reserve; ++i) pl.pool_ids.push_back(row[it.start + it.n_pages - 1]);
                cap += tail_reserve;
            }
        }
        pl.item_pool_cap.push_back(cap);
        pl.item_num_pages.push_back(it.n_pages);
        pl.item_req_off.push_back((int32_t)pl.item_req_ids.size());
        pl.item_page_off.push_back((int32_t)pl.item_page_ids.size());
        pl.item_page_start.push_back(it.start);
        pl.item_kv_len.push_back(it.kv_len);
        item_heads.push_back(it.heads_per_wg);
    }
    pl.req_slot_off.assign(1, 0);
    for (int32_t r = 0; r < B; ++r) {
        for (int32_t s : req_slots[r]) pl.req_slot_ids.push_back(s);
        pl.req_slot_off.push_back((int32_t)pl.req_slot_ids.size());
        if (req_slots[r].size() > 1) pl.merge_req.push_back(r);
    }

    // ---- entries: row blocks + tiles -------------------------------------------------------
    struct E { int32_t item, row_begin, n_rows, tile; };
    std::vector<E> es;
    std::vector<char> item_wave;
    for (int32_t k = 0; k < n_items; ++k) item_wave.push_back(items[perm[k]].wave ? 1 : 0);
    for (int32_t k = 0; k < n_items; ++k) {
        int32_t n_req = pl.item_req_off[k + 1] - pl.item_req_off[k];
        int32_t rows = n_req * G;
        const int32_t len = pl.item_kv_len[k];
        const int32_t wkv = item_wave[k] ? INT32_MAX : 0;
        int32_t tile = o.force_tile >= 0 ? o.force_tile : select_tile(rows, len, wkv, packed_min);
        int32_t m = kTiles[tile].m;
        int32_t blocks = (rows + m - 1) / m;
        int32_t per = (rows + blocks - 1) / blocks;
        if (o.force_tile < 0 && blocks > 1 && is_packed_tile(tile)) {
            // equal blocks may fit a smaller tile than the largest one
            int32_t t2 = select_tile(per, len, 0, packed_min);
            if (is_packed_tile(t2) && kTiles[t2].m >= per) { tile = t2; m = kTiles[t2].m; }
        }
        for (int32_t rb = 0; rb < rows; rb += per)
            es.push_back({k, rb, std::min(per, rows - rb), tile});
    }
    // launch order: longest-running first, priced as the cuts were (bytes; a packed workgroup
    // a quarter above its bytes)
    auto heads_of = [&](const E &x) {
        return is_packed_tile(x.tile) || x.tile == TILE_WAVE16 || dual ? 1 : item_heads[x.item];
    };
    auto cost = [&](const E &x) {
        const int64_t len = pl.item_kv_len[x.item];
        return is_packed_tile(x.tile) ? 5 * len : 4 * heads_of(x) * len;
    };
    std::stable_sort(es.begin(), es.end(),
                     [&](const E &a, const E &c) { return cost(a) > cost(c); });
    if (dual)       // the packed tiles' kernel takes the first units, the 16-row kernel the rest
        std::stable_partition(es.begin(), es.end(), [&](const E &x) { return is_packed_tile(x.tile); });
    std::memset(&pl.stats, 0, sizeof pl.stats);
    std::vector<int32_t> unit_item, wave_item_of;       // the item of every unit / wavefront item
    for (const E &e : es) {
        pl.entry_item.push_back(e.item);
        pl.entry_row_begin.push_back(e.row_begin);
        pl.entry_num_rows.push_back(e.n_rows);
        pl.entry_tile.push_back(e.tile);
        pl.entry_heads_per_wg.push_back(heads_of(e));
        DevEntry d;
        d.req_off = pl.item_req_off[e.item];
        d.n_req = pl.item_req_off[e.item + 1] - pl.item_req_off[e.item];
        d.page_off = pl.item_pool_base[e.item];
        d.n_pages = pl.item_num_pages[e.item];
        d.kv_len = pl.item_kv_len[e.item];
        d.row_begin = e.row_begin;
        d.n_rows = e.n_rows;
        d.tile = e.tile;
        pl.stats.tile_histogram[e.tile]++;
        if (e.tile == TILE_WAVE16) {
            // one wavefront item per KV head
            for (int32_t h = 0; h < pl.Hkv; ++h) {
                DevWaveItem w;
                std::memset(&w, 0, sizeof w);
                w.req_off = d.req_off; w.n_req = d.n_req; w.page_off = d.page_off;
                w.n_pages = d.n_pages; w.kv_len = d.kv_len; w.row_begin = d.row_begin;
                w.n_rows = d.n_rows; w.kvh = h;
                w.req0 = pl.item_req_ids[d.req_off];
                w.slot0 = pl.item_req_slot[d.req_off];
                w.page0 = pl.pool_ids[d.page_off];
                w.page1 = pl.pool_ids[d.page_off + std::min(1, d.n_pages - 1)];
                wave_item_of.push_back(e.item);
                pl.wave_items.push_back(w);
            }
            continue;
        }
        // workgroups of this entry: one per KV head for packed tiles; the 16-row tiles run a
        // head per 256-thread half, so one per pair of KV heads unless the cut asked for one
        const int32_t per_wg = heads_of(e);
        for (int32_t h0 = 0; h0 < pl.Hkv; h0 += per_wg) {
            DevUnit u;
            std::memset(&u, 0, sizeof u);
            u.e = d;
            u.kvh0 = h0;
            u.n_heads = std::min(per_wg, pl.Hkv - h0);
            int32_t *unit_pages[kUnitPages] = {&u.page0, &u.page1, &u.page2, &u.page3,
                                               &u.page4, &u.page5, &u.page6, &u.page7};
            int32_t *unit_reqs[kUnitReqs] = {&u.req0, &u.req1, &u.req2, &u.req3};
            for (int32_t i = 0; i < kUnitPages; ++i)
                *unit_pages[i] = pl.pool_ids[d.page_off + std::min(i, d.n_pages - 1)];
            for (int32_t i = 0; i < kUnitReqs; ++i)
                *unit_reqs[i] = pl.item_req_ids[d.req_off + std::min(i, d.n_req - 1)];
            unit_item.push_back(e.item);
            pl.units.push_back(u);
        }
    }
    pl.queue_begin = (int32_t)pl.units.size();
    pl.queue_workers = 0;
    pl.dual = dual;
    pl.stream_begin = 0;
    while (pl.stream_begin < (int32_t)pl.units.size() && is_packed_tile(pl.units[pl.stream_begin].e.tile))
        ++pl.stream_begin;
    const int32_t cus = o.num_cus > 0 ? o.num_cus : 256;
    if (dual) {
        // no queue: the hardware hands the 16-row workgroups to half CUs as they free up
    } else if (!pl.wave_items.empty()) {
        // Static schedule of a launch with wavefront items: `cus` persistent workgroups.  The
        // workgroup-level units go to the workgroup that is free first, longest first, by the
        // run-time model; then the wavefront items go, longest first, to the wavefront that is
        // free first, a workgroup's eight wavefronts starting when its units are done.
        auto unit_ns = [&](const DevUnit &u) {
            if (is_packed_tile(u.e.tile))
                return (u.e.n_rows <= 64 ? c0q : c0p) + (u.e.n_rows <= 64 ? c1q : c1p) * (int64_t)u.e.kv_len;
            return c0s + c1s * u.n_heads * (int64_t)u.e.kv_len;
        };
        const int32_t n_workers = cus;
        typedef std::pair<int64_t, int32_t> Slot;                 // (free at, index)
        std::vector<int32_t> order(pl.units.size());
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            return unit_ns(pl.units[x]) > unit_ns(pl.units[y]);
        });
        // The launch, if it packed perfectly.  Units are packed first-fit (longest first) into
        // workgroups of that capacity rather than spread evenly: workgroups then either run units
        // for the whole launch or walk wavefront items from its start, so that the streams of the
        // items and the (often compute-bound) packed tiles share the memory system all the time
        // instead of one after the other.
        int64_t total_ns = 0;
        for (const DevUnit &u : pl.units) total_ns += unit_ns(u);
        for (const DevWaveItem &w : pl.wave_items) total_ns += (c0w + c1w * (int64_t)w.kv_len) / 8;
        const int64_t ideal = (total_ns + n_workers - 1) / n_workers;
        std::vector<std::vector<int32_t>> wg_units(n_workers);
        std::vector<int64_t> wg_free(n_workers, 0);
        for (int32_t x : order) {
            const int64_t t = unit_ns(pl.units[x]);
            int32_t best = -1;
            for (int32_t w = 0; w < n_workers && best < 0; ++w)
                if (wg_free[w] + t <= std::max(ideal, t)) best = w;
            if (best < 0)
                best = (int32_t)(std::min_element(wg_free.begin(), wg_free.end()) - wg_free.begin());
            wg_units[best].push_back(x);
            wg_free[best] += t;
        }
        std::priority_queue<Slot, std::vector<Slot>, std::greater<Slot>> free_wave;
        for (int32_t w = 0; w < n_workers; ++w)
            for (int32_t v = 0; v < 8; ++v) free_wave.push({wg_free[w], w * 8 + v});
        std::vector<int32_t> worder(pl.wave_items.size());
        std::iota(worder.begin(), worder.end(), 0);
        std::stable_sort(worder.begin(), worder.end(), [&](int32_t x, int32_t y) {
            return pl.wave_items[x].kv_len > pl.wave_items[y].kv_len;
        });
        std::vector<std::vector<int32_t>> wave_lists((size_t)n_workers * 8);
        for (int32_t x : worder) {
            Slot sl = free_wave.top();
            free_wave.pop();
            wave_lists[sl.second].push_back(x);
            sl.first += c0w + c1w * (int64_t)pl.wave_items[x].kv_len;
            free_wave.push(sl);
        }
        // lay units and items out in that order
        std::vector<DevUnit> units2;
        std::vector<int32_t> unit_item2;
        std::vector<DevWaveItem> items2;
        std::vector<int32_t> wave_item_of2;
        pl.workers.assign(n_workers, DevWorker{});
        for (int32_t w = 0; w < n_workers; ++w) {
            DevWorker &wk = pl.workers[w];
            std::memset(&wk, 0, sizeof wk);
            wk.unit_begin = (int32_t)units2.size();
            for (int32_t x : wg_units[w]) {
                units2.push_back(pl.units[x]);
                unit_item2.push_back(unit_item[x]);
            }
            wk.unit_end = (int32_t)units2.size();
            for (int32_t v = 0; v < 8; ++v) {
                wk.item_off[v] = (int32_t)items2.size();
                for (int32_t x : wave_lists[(size_t)w * 8 + v]) {
                    items2.push_back(pl.wave_items[x]);
                    wave_item_of2.push_back(wave_item_of[x]);
                }
            }
            wk.item_off[8] = (int32_t)items2.size();
        }
        pl.units.swap(units2);
        unit_item.swap(unit_item2);
        pl.wave_items.swap(items2);
        wave_item_of.swap(wave_item_of2);
        pl.queue_begin = (int32_t)pl.units.size();
    } else {
        // Long 16-row units at the end of a launch of many rounds are not workgroups of their own: as
        // many persistent workgroups as there are CUs take them from a queue in the same order,
        // which saves a workgroup launch per unit (C5: 3 %).  Short units stay workgroups: drawing
        // from the queue costs an atomic's round trip per unit (C4 was 1 % slower with a queue).
        int32_t last_packed = -1;
        for (int32_t u = 0; u < (int32_t)pl.units.size(); ++u)
            if (is_packed_tile(pl.units[u].e.tile)) last_packed = u;
        const int32_t queued = (int32_t)pl.units.size() - (last_packed + 1);
        int64_t token_heads = 0;
        for (int32_t u = last_packed + 1; u < (int32_t)pl.units.size(); ++u)
            token_heads += (int64_t)pl.units[u].e.kv_len * pl.units[u].n_heads;
        if (queued >= 2 * cus && token_heads >= (int64_t)4096 * queued && o.force_tile < 0) {
            pl.queue_begin = last_packed + 1;
            pl.queue_workers = cus;
        }
    }
    // CSR: the units and the wavefront items of each item (for pat_plan_advance)
    {
        std::vector<std::vector<int32_t>> of_item(n_items), waves_of_item(n_items);
        for (size_t x = 0; x < unit_item.size(); ++x) of_item[unit_item[x]].push_back((int32_t)x);
        for (size_t x = 0; x < wave_item_of.size(); ++x) waves_of_item[wave_item_of[x]].push_back((int32_t)x);
        pl.item_unit_off.assign(1, 0);
        pl.item_wave_off.assign(1, 0);
        for (int32_t k = 0; k < n_items; ++k) {
            for (int32_t x : of_item[k]) pl.item_units.push_back(x);
            pl.item_unit_off.push_back((int32_t)pl.item_units.size());
            for (int32_t x : waves_of_item[k]) pl.item_waves.push_back(x);
            pl.item_wave_off.push_back((int32_t)pl.item_waves.size());
        }
    }

    // ---- merge fused into the forward launch ----------------------------------------------------
    // (plain single-kernel launches only: no unit queue, no wavefront items, no second stream)
    std::vector<int32_t> merge_expected(pl.merge_req.size(), 0);
    {
        std::vector<int32_t> midx_of_req(B, -1);
        for (size_t i = 0; i < pl.merge_req.size(); ++i) midx_of_req[pl.merge_req[i]] = (int32_t)i;
        pl.item_req_midx.resize(pl.item_req_ids.size());
        for (size_t i = 0; i < pl.item_req_ids.size(); ++i)
            pl.item_req_midx[i] = pl.item_req_slot[i] >= 0 ? midx_of_req[pl.item_req_ids[i]] : -1;
        // arrivals that complete a task (request, KV head): one per entry that holds rows of the
        // request (the entry's workgroup for that head signals once per request it touches)
        for (size_t e = 0; e < pl.entry_item.size(); ++e) {
            const int32_t k = pl.entry_item[e], rb = pl.entry_row_begin[e], n = pl.entry_num_rows[e];
            for (int32_t pos = rb / G; pos <= (rb + n - 1) / G; ++pos) {
                const int32_t mi = pl.item_req_midx[pl.item_req_off[k] + pos];
                if (mi >= 0) ++merge_expected[mi];
            }
        }
        const bool plain = pl.queue_workers == 0 && pl.workers.empty() && !pl.dual;
        pl.fuse_mode = 0;
        // Measured on MI355X: slower than the merge kernel on every benchmark shape (C2 32.8 against
        // 23.0 us per step, C3 126 against 110, C4 211 against 200).  A workgroup has to wait for
        // its partial stores to be acknowledged from memory and then for an atomic's round trip
        // before it may leave, with nothing in flight meanwhile, and the merge's own two dependent
        // fetches come on top; the kernel boundary it replaces costs less than that chain.  So the
        // planner uses it only where the caller asks for it.
        if (o.fused_merge > 0 && plain && !pl.merge_req.empty() && o.force_tile != TILE_VALU16)
            pl.fuse_mode = (int32_t)pl.units.size() <= cus ? 2 : 1;
    }

    // ---- device image ----------------------------------------------------------------------
    DevLayout &L = pl.layout;
    size_t off = 0;
    auto place = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    L.units = place(pl.units.size() * sizeof(DevUnit));
    L.req_ids = place(pl.item_req_ids.size() * 4);
    L.req_slot = place(pl.item_req_slot.size() * 4);
    L.page_ids = place((pl.pool_ids.size() + kPageIdSlack) * 4);   // zero slack (staging starts zeroed)
    L.merge_rec = place(pl.merge_req.size() * kMergeRecInts * 4);
    L.req_slot_off = place(pl.req_slot_off.size() * 4);
    L.req_slot_ids = place(pl.req_slot_ids.size() * 4);
    L.queue_ctr = place(256);
    L.req_midx = place(pl.item_req_midx.size() * 4);
    L.merge_state = place(pl.merge_req.size() * (size_t)pl.Hkv * 4);
    L.workers = place(pl.workers.size() * sizeof(DevWorker));
    L.wave_items = place(pl.wave_items.size() * sizeof(DevWaveItem));
    L.total = std::max<size_t>(off, 256);
    pl.staging.assign(L.total, 0);
    auto put = [&](size_t at, const void *src, size_t bytes) {
        if (bytes) std::memcpy(pl.staging.data() + at, src, bytes);
    };
    put(L.units, pl.units.data(), pl.units.size() * sizeof(DevUnit));
    put(L.req_ids, pl.item_req_ids.data(), pl.item_req_ids.size() * 4);
    put(L.req_slot, pl.item_req_slot.data(), pl.item_req_slot.size() * 4);
    put(L.page_ids, pl.pool_ids.data(), pl.pool_ids.size() * 4);
    put(L.req_slot_off, pl.req_slot_off.data(), pl.req_slot_off.size() * 4);
    put(L.req_midx, pl.item_req_midx.data(), pl.item_req_midx.size() * 4);
    {
        // task state words start as "abandoned" where only the last arriver merges
        std::vector<int32_t> st(pl.merge_req.size() * (size_t)pl.Hkv, pl.fuse_mode == 1 ? kFuseAbandoned : 0);
        put(L.merge_state, st.data(), st.size() * 4);
    }
    put(L.workers, pl.workers.data(), pl.workers.size() * sizeof(DevWorker));
    put(L.wave_items, pl.wave_items.data(), pl.wave_items.size() * sizeof(DevWaveItem));
    {
        // device copy of the merge lists: bit 30 marks partials the packed tiles wrote with the
        // head dimension in their internal order (see kPartialPermutedBit)
        std::vector<char> permuted((size_t)n_slots, 0);
        for (size_t e = 0; e < pl.entry_item.size(); ++e) {
            if (!is_packed_tile(pl.entry_tile[e])) continue;
            const int32_t k = pl.entry_item[e];
            for (int32_t i = pl.item_req_off[k]; i < pl.item_req_off[k + 1]; ++i)
                if (pl.item_req_slot[i] >= 0) permuted[pl.item_req_slot[i]] = 1;
        }
        std::vector<int32_t> dev_ids(pl.req_slot_ids);
        for (int32_t &x : dev_ids)
            if (permuted[x]) x |= kPartialPermutedBit;
        put(L.req_slot_ids, dev_ids.data(), dev_ids.size() * 4);
        std::vector<int32_t> recs(pl.merge_req.size() * kMergeRecInts, 0);
        for (size_t i = 0; i < pl.merge_req.size(); ++i) {
            const int32_t r = pl.merge_req[i];
            const int32_t s0 = pl.req_slot_off[r], n = pl.req_slot_off[r + 1] - s0;
            int32_t *rec = recs.data() + i * kMergeRecInts;
            rec[0] = r;
            rec[1] = n;
            rec[2] = s0;
            rec[3] = merge_expected[i];
            for (int32_t k = 0; k < std::min<int32_t>(n, kMergeInline); ++k) rec[4 + k] = dev_ids[s0 + k];
        }
        put(L.merge_rec, recs.data(), recs.size() * 4);
    }

    // ---- workspace: fp32 partial O [slots][Hq][d], then partial LSE [slots][Hq] ------------
    pl.ws_part_o = 0;
    pl.ws_part_lse = align_up((size_t)n_slots * pl.Hq * pl.d * 4, 256);
    size_t ws = pl.ws_part_lse + align_up((size_t)n_slots * pl.Hq * 4, 256);

    pat_plan_stats &s = pl.stats;
    s.num_nodes = (int32_t)f.nodes.size();
    s.num_packs = (int32_t)packs.size();
    s.num_merged_children = pk.merged_children;
    s.num_items = n_items;
    s.num_entries = (int32_t)pl.entry_item.size();
    s.num_workgroups = (int32_t)(pl.units.size() + pl.wave_items.size());
    s.num_wave_items = (int32_t)pl.wave_items.size();
    s.num_workers = (int32_t)pl.workers.size();
    s.fused_merge = pl.fuse_mode;
    s.num_slots = n_slots;
    s.num_merge_requests = (int32_t)pl.merge_req.size();
    s.unique_kv_tokens = unique_tokens;
    s.total_kv_tokens = 0;
    for (int32_t r = 0; r < B; ++r) s.total_kv_tokens += b.kv_lens[r];
    s.plan_device_bytes = (int64_t)L.total;
    s.workspace_bytes = (int64_t)std::max<size_t>(ws, 256);
    return PAT_OK;
}

// Lazy update: grow the last item of every request whose kv_len grew.  Two passes: nothing is
// touched unless every request can be served.
int advance_plan(pat_plan_s &pl, const int32_t *new_kv_lens, const int32_t *block_tables, int32_t W)
{
    const int32_t B = pl.B, P = pl.P;
    for (int32_t r = 0; r < B; ++r) {
        const int32_t old_len = pl.kv_lens[r], new_len = new_kv_lens[r];
        if (new_len == old_len) continue;
        if (new_len < old_len) return PAT_ERR_PLAN_STALE;
        const int32_t old_pages = (old_len + P - 1) / P, new_pages = (new_len + P - 1) / P;
        if (new_pages > W) return PAT_ERR_BAD_KV_LEN;
        const int32_t k = pl.req_tail_item[r];
        if (k < 0) return PAT_ERR_PLAN_STALE;                  // ends inside shared pages
        const int32_t n = pl.item_num_pages[k];
        if (n + (new_pages - old_pages) > pl.item_pool_cap[k]) return PAT_ERR_PLAN_STALE;
        const int32_t *row = block_tables + (int64_t)r * W;
        if (row[old_pages - 1] != pl.pool_ids[pl.item_pool_base[k] + n - 1]) return PAT_ERR_PLAN_STALE;
        for (int32_t i = old_pages; i < new_pages; ++i)
            if (row[i] < 0 || row[i] >= pl.num_pages) return PAT_ERR_BAD_PAGE_ID;
    }
    unsigned char *img = pl.staging.data();
    int32_t *img_pages = reinterpret_cast<int32_t *>(img + pl.layout.page_ids);
    DevUnit *img_units = reinterpret_cast<DevUnit *>(img + pl.layout.units);
    DevWaveItem *img_waves = reinterpret_cast<DevWaveItem *>(img + pl.layout.wave_items);
    for (int32_t r = 0; r < B; ++r) {
        const int32_t old_len = pl.kv_lens[r], new_len = new_kv_lens[r];
        if (new_len == old_len) continue;
        const int32_t old_pages = (old_len + P - 1) / P, new_pages = (new_len + P - 1) / P;
        const int32_t k = pl.req_tail_item[r];
        const int32_t base = pl.item_pool_base[k];
        const int32_t *row = block_tables + (int64_t)r * W;
        int32_t n = pl.item_num_pages[k];
        for (int32_t i = old_pages; i < new_pages; ++i, ++n) {
            pl.pool_ids[base + n] = row[i];
            img_pages[base + n] = row[i];
        }
        // unused reserve slots keep a valid id (the kernels prefetch ids past an entry's end)
        for (int32_t i = n; i < pl.item_pool_cap[k]; ++i) {
            pl.pool_ids[base + i] = pl.pool_ids[base + n - 1];
            img_pages[base + i] = pl.pool_ids[base + n - 1];
        }
        pl.item_num_pages[k] = n;
        pl.item_kv_len[k] += new_len - old_len;
        pl.kv_lens[r] = new_len;
        pl.stats.unique_kv_tokens += new_len - old_len;
        pl.stats.total_kv_tokens += new_len - old_len;
        for (int32_t x = pl.item_unit_off[k]; x < pl.item_unit_off[k + 1]; ++x) {
            DevUnit &u = pl.units[pl.item_units[x]];
            u.e.n_pages = n;
            u.e.kv_len = pl.item_kv_len[k];
            int32_t *unit_pages[kUnitPages] = {&u.page0, &u.page1, &u.page2, &u.page3,
                                               &u.page4, &u.page5, &u.page6, &u.page7};
            for (int32_t i = 0; i < kUnitPages; ++i)
                *unit_pages[i] = pl.pool_ids[base + std::min(i, n - 1)];
            img_units[pl.item_units[x]] = u;
        }
        for (int32_t x = pl.item_wave_off[k]; x < pl.item_wave_off[k + 1]; ++x) {
            DevWaveItem &w = pl.wave_items[pl.item_waves[x]];
            w.n_pages = n;
            w.kv_len = pl.item_kv_len[k];
            w.page0 = pl.pool_ids[base];
            w.page1 = pl.pool_ids[base + std::min(1, n - 1)];
            img_waves[pl.item_waves[x]] = w;
        }
        pl.view_dirty = true;
    }
    return PAT_OK;
}

// Rebuild the exact page CSR of the exported view from the pool after pat_plan_advance().
void refresh_view(pat_plan_s &pl)
{
    if (!pl.view_dirty) return;
    const int32_t n_items = (int32_t)pl.item_num_pages.size();
    pl.item_page_off.assign(1, 0);
    pl.item_page_ids.clear();
    for (int32_t k = 0; k < n_items; ++k) {
        for (int32_t i = 0; i < pl.item_num_pages[k]; ++i)
            pl.item_page_ids.push_back(pl.pool_ids[pl.item_pool_base[k] + i]);
        pl.item_page_off.push_back((int32_t)pl.item_page_ids.size());
    }
    pl.view_dirty = false;
}

}  // namespace pat
