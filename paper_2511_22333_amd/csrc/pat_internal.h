// Internal structures shared by the planner (host) and the launcher.  Not part of the ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "pat.h"

namespace pat {

// Tile ids of the forward kernel family.  m = query rows held by one workgroup, n = KV tokens
// the workgroup consumes per pipeline stage (sec. "Multi-tile Kernel": the (m, n) pairs are
// re-derived for gfx950 rather than taken from the paper's A100 table).
enum TileId : int32_t {
    TILE_VALU16 = 0,     // rows <= 16, VALU dot products, 4 tokens per stage (reference tile)
    TILE_STREAM16 = 1,   // rows <= 16, MFMA, four independent wave streams of 32 tokens
    TILE_WAVE16 = 2,     // rows <= 16, MFMA, one wavefront per (entry, KV head), 32-token stages
    TILE_PACKED64 = 3,
    TILE_PACKED128 = 4,
    NUM_TILES = 5
};

struct TileInfo {
    int32_t m, n;
    bool available;      // a kernel exists for it
};
const TileInfo &tile_info(int id);

// Packed tiles keep the head dimension in the order d' = 16 * (d % 8) + d / 8 and write their fp32
// partials that way (their registers hold four consecutive d', so rows go out as 16-byte stores
// with no transpose).  The merge lists on the device carry this bit on such slots.
constexpr int32_t kPartialPermutedBit = 1 << 30;

// One record per request that has more than one partial, 128 bytes: the request, the number of
// its partials, where its full list starts in the slot-id list, and the first kMergeInline slot
// ids themselves (bit 30 as above) -- so the merge kernel reaches the partials in two dependent
// fetches instead of four.
constexpr int kMergeRecInts = 32;
// state word of a fused-merge task: arrivals so far, and who takes the merge
constexpr int32_t kFuseCountMask = (1 << 20) - 1, kFuseClaimed = 1 << 29, kFuseAbandoned = 1 << 30;
constexpr int kMergeInline = 28;

// Zero page ids the planner appends to the device page-id list: the kernels prefetch ids a few
// tiles past the end of an entry without clamping.
constexpr int kPageIdSlack = 64;

// One entry: a block of rows of one work item (all KV heads).
struct DevEntry {
    int32_t req_off;      // first request of the item in req_ids / req_slot
    int32_t n_req;        // requests in the item
    int32_t page_off;     // first page of the item in page_ids
    int32_t n_pages;
    int32_t kv_len;       // valid tokens (only the last page may be partial)
    int32_t row_begin;    // first row of this block; row = req_pos * G + head_in_group
    int32_t n_rows;       // rows in this block (<= tile m)
    int32_t tile;
};

// One workgroup's work, 128 bytes, fetched with two scalar loads: an entry, the KV head(s) the
// workgroup serves, and copies of the entry's first page ids and request ids, so that the first
// K/V and q loads depend on this record alone (every further dependent fetch at start-up costs a
// round trip through a memory system the whole chip is loading).  Packed tiles run all 512
// threads on one head; the 16-row tiles run two heads side by side, one per 256-thread half
// (n_heads = 1 leaves the second half idle).
constexpr int kUnitPages = 8;     // page ids 0..7 of the entry (past its end: its last page id)
constexpr int kUnitReqs = 4;      // request ids 0..3 of the entry (past its end: its last request)
struct DevUnit {
    DevEntry e;
    int32_t kvh0;         // first KV head
    int32_t n_heads;      // 1 or 2
    int32_t pad0[2];
    // named fields rather than arrays: the kernels keep the record in scalar registers
    int32_t page0, page1, page2, page3, page4, page5, page6, page7;
    int32_t req0, req1, req2, req3;
    int32_t pad1[8];
};
static_assert(sizeof(DevUnit) == 128, "DevUnit is one 128-byte record");

// One item of TILE_WAVE16: an entry's rows against one KV head, walked by a single wavefront.
// 64 bytes; carries the entry's first two page ids (index 1 clamped to the last page) and, for
// entries of one request, the request id and its partial slot, so that the first loads need this
// record only.
struct DevWaveItem {
    int32_t req_off, n_req, page_off, n_pages, kv_len, row_begin, n_rows, kvh;
    int32_t req0, slot0, page0, page1;
    int32_t pad[4];
};
static_assert(sizeof(DevWaveItem) == 64, "DevWaveItem is one 64-byte record");

// One persistent workgroup of a launch that holds wavefront items: first the workgroup-level
// units [unit_begin, unit_end), one after the other, then wavefront w walks the wavefront items
// [item_off[w], item_off[w + 1]).  64 bytes.
struct DevWorker {
    int32_t unit_begin, unit_end;
    int32_t item_off[9];
    int32_t pad[5];
};
static_assert(sizeof(DevWorker) == 64, "DevWorker is one 64-byte record");

// Offsets (in bytes from the start of the uploaded buffer) of the device arrays.
struct DevLayout {
    size_t units = 0, req_ids = 0, req_slot = 0, page_ids = 0;
    size_t merge_rec = 0, req_slot_off = 0, req_slot_ids = 0;
    size_t queue_ctr = 0;            // two counters of the 16-row unit queue (own 256 bytes)
    size_t workers = 0, wave_items = 0;
    size_t req_midx = 0, merge_state = 0;     // fused merge: see pat_plan_s::fuse_mode
    size_t total = 0;
};

}  // namespace pat

struct pat_plan_s {
    // problem
    int32_t B = 0, Hq = 0, Hkv = 0, d = 0, P = 0, dtype = 0, num_pages = 0;
    pat_plan_opts opts{};
    // schedule (host)
    std::vector<int32_t> item_req_off, item_req_ids, item_req_slot;
    std::vector<int32_t> item_page_off, item_page_ids, item_page_start, item_kv_len;
    std::vector<int32_t> req_slot_off, req_slot_ids;
    std::vector<int32_t> entry_item, entry_row_begin, entry_num_rows, entry_tile;
    std::vector<int32_t> entry_heads_per_wg;
    // page-id pool as the device sees it: item k owns pool_ids[item_pool_base[k] .. +
    // item_pool_cap[k]), of which the first item_num_pages[k] are in use; the rest (only the
    // tail item of a request has any) is room for pat_plan_advance() and holds valid ids
    std::vector<int32_t> pool_ids, item_pool_base, item_pool_cap, item_num_pages;
    std::vector<int32_t> item_unit_off, item_units;   // CSR: the workgroups of each item
    std::vector<int32_t> kv_lens, req_tail_item;      // current length; own last item or -1
    bool view_dirty = false;                          // item_page_off/ids lag behind the pool
    std::mutex view_mutex;                            // pat_plan_export() brings the view up to date under it
    std::vector<int32_t> merge_req;              // requests with more than one partial
    std::vector<pat::DevUnit> units;             // one per workgroup, launch order
    // Units [queue_begin, units.size()) are 16-row units taken from a queue by queue_workers
    // persistent workgroups; queue_begin == units.size(): every unit is a workgroup of its own.
    int32_t queue_begin = 0, queue_workers = 0;
    // Two-kernel launches: units [0, stream_begin) are packed tiles (512-thread workgroups on the
    // caller's stream), units [stream_begin, units.size()) 16-row tiles of one KV head each
    // (256-thread workgroups on side_stream, which forks from and joins the caller's stream).
    bool dual = false;
    int32_t stream_begin = 0;
    void *side_stream = nullptr, *ev_fork = nullptr, *ev_join = nullptr;   // created by pat_plan_upload
    // Merge fused into the forward launch.  0: off.  1: every (request, KV head) task has an
    // arrival counter; the workgroup whose unit completes it merges the request.  2 (launches of
    // one round): workgroups that are done also claim tasks in order and wait, bounded, for them.
    // item_req_midx runs parallel to item_req_ids: index of the request's merge record or -1;
    // a merge record's int 3 holds the arrivals that complete a task of that request.
    int32_t fuse_mode = 0;
    std::vector<int32_t> item_req_midx;
    // Launches with wavefront items run as `workers.size()` persistent workgroups instead.
    std::vector<pat::DevWorker> workers;
    std::vector<pat::DevWaveItem> wave_items;
    std::vector<int32_t> item_wave_off, item_waves;   // CSR: the wavefront items of each item
    pat_plan_stats stats{};
    // device copy
    pat::DevLayout layout;
    std::vector<unsigned char> staging;          // host image of the device buffer
    void *device_buf = nullptr;                  // caller-owned, set by pat_plan_upload
    size_t ws_part_o = 0, ws_part_lse = 0;       // byte offsets inside the workspace
};
