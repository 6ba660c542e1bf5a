// Forward tiles TILE_PACKED64 / TILE_PACKED128: up to 128 query rows that share one KV range
// (sec. "Multi-tile Kernel": the packed queries of a prefix node x the node's keys, K and V
// staged once in shared memory for all of them).
//
// All eight wavefronts of the workgroup load AND compute.  A 64-token tile of K and V is staged
// in LDS once; a computing wavefront owns the 32 rows of one row group and the 32 tokens of one
// token half of every tile, with its own online-softmax state.  With four row groups (128
// rows) wavefront w takes row group w % 4 and token half w / 4: the two wavefronts of a row
// group sit on the same SIMD, so while one waits for its MFMA chain, its LDS operands or the
// exponentials of its softmax, the other one issues -- the matrix pipe, the vector ALU and the
// LDS pipe overlap through the hardware's wavefront interleaving instead of a hand-made
// instruction order.  With two row groups (64 rows) wavefronts 0..3 compute, one per SIMD, and
// 4..7 only load.  The two states of a row group are combined through LDS at the end (sec.
// "Output Merge" applied inside the workgroup).
//
//   S^T[token][row] = K . Q^T       8 x v_mfma_f32_32x32x16 per tile and wavefront
//   O^T[d'][row]   += V^T . P^T     8 x v_mfma_f32_32x32x16
//
// LDS operand buffers (two, tile t in buffer t % 2), layouts as the MFMA operands want them:
//   Ks[token 0..63][d 0..127]        row pitch 272 B
//   Vt[d' 0..127][position 0..63]    row pitch 144 B, d' = 16 (d % 8) + d / 8, and position
//                                    8 gamma + kappa holds the token listed below
// Loading: every thread fetches four 16-byte pieces of each tile into registers (two tiles in
// flight, inline-asm loads with explicit waits, page ids through the scalar cache one tile
// ahead) and stores them to LDS one tile ahead of the compute; V goes through a 4x8 16-bit
// transpose in registers on the way.  One LDS-only barrier per tile.
#pragma once
#include <type_traits>

#include "pat_common.hip.h"
#include "pat_lds_barrier.hip.h"

namespace pat {

namespace pk {
constexpr int kTileTokens = 64;             // tokens per tile (four pages)
constexpr int kKsPitch = 136;               // halves per K row in LDS (272 bytes)
constexpr int kVtPitch = 72;                // halves per V^T row in LDS (64 tokens + 8 pad)
constexpr int kOsPitch = 132;               // floats per epilogue row
constexpr int kKBytes = kTileTokens * kKsPitch * 2;          // 17408
constexpr int kVBytes = kHeadDim * kVtPitch * 2;             // 18432
constexpr int kBufBytes = kKBytes + kVBytes;                 // 35840
constexpr int kXchgBytes = 64 * 64 * 4 + 2 * 64 * 4;         // one wavefront's state: acc, m, l
constexpr int kParkBytes = 4 * 5 * 64 * 4;                   // epilogue destinations, parked
static_assert(2 * kBufBytes + kParkBytes <= kFwdSmemBytes, "LDS budget");
static_assert(4 * kXchgBytes <= 2 * kBufBytes, "state exchange aliases the tile buffers");
static_assert(4 * 16 * kOsPitch * 4 <= 2 * kBufBytes, "epilogue buffer aliases the tile buffers");
static_assert(4 * 5 <= kPageIdSlack, "ids are requested up to four tiles past the entry");
}  // namespace pk

// Position kappa (0..7) of contraction group gamma (0..7) of a 64-token tile holds token
//   32*sub + 16*n + 8*(kappa/4) + 4*h + kappa%4,   gamma = 4*sub + 2*n + h
// (32-token half `sub`, MFMA `n` of that half, lane half `h`).  This is the order in which the
// S^T accumulator holds its values, so P needs no shuffling before the second product.  All
// eight tokens of a group lie in page gamma/2 of the tile.

// The K and V loads are issued through inline asm and waited for with explicit s_waitcnt: the
// compiler's own wait insertion does not follow loads across loop iterations and would drain
// everything in flight (vmcnt(0)) before every staging step.  Loads return in issue order, so
// "at most N loads outstanding" means everything older than the last N has landed.
//
// Their destinations are FIXED registers, v224..v255, which the kernel keeps out of the
// compiler's hands (see kVgprLimitAttr).  Had the loads
// ordinary asm outputs, the register allocator would be free to copy or move them while they
// are still in flight -- it believes an asm statement's outputs are there when the statement
// ends -- and under this tile's register pressure it does.  Slot s, load i lives in
// v[224 + 16 s + 4 i .. + 3]; after the wait the values are copied out with v_mov.
// Value of the kernel's VGPR-limit attribute that makes the compiler stop at v223: it counts the
// unified (VGPR + AGPR) register file of this GPU family in halves.  The build checks the
// generated ISA for what the compiler actually did with it.
constexpr int kVgprLimitAttr = 112;
constexpr int kRingBase = 224;
// The address is a wavefront-uniform base (scalar registers) plus a 32-bit byte offset per lane.
template <int SLOT, int I>
__device__ __forceinline__ void ring_load(const uint16_t *base, uint32_t lane_off)
{
    constexpr int R = kRingBase + 16 * SLOT + 4 * I;
    asm volatile("global_load_dwordx4 v[%2:%3], %0, %1 nt" ::"v"(lane_off), "s"(base), "n"(R), "n"(R + 3)
                 : "memory");
}
template <int SLOT, int I>
__device__ __forceinline__ u32x4 ring_read()
{
    constexpr int R = kRingBase + 16 * SLOT + 4 * I;
    u32x4 x;
    asm volatile("v_mov_b32 %0, v[%4]\n\tv_mov_b32 %1, v[%5]\n\tv_mov_b32 %2, v[%6]\n\tv_mov_b32 %3, v[%7]"
                 : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3])
                 : "n"(R), "n"(R + 1), "n"(R + 2), "n"(R + 3)
                 : "memory");
    return x;
}
// Straight from the ring to LDS (K), or through the byte permute that starts V's transpose,
// without a copy into registers of the compiler's choosing.
template <int SLOT, int I, int OFFSET>
__device__ __forceinline__ void ring_store_lds(uint32_t lds_addr)
{
    constexpr int R = kRingBase + 16 * SLOT + 4 * I;
    static_assert(OFFSET >= 0 && OFFSET < 65536, "16-bit offset field");
    asm volatile("ds_write_b128 %0, v[%1:%2] offset:%3" ::"v"(lds_addr), "n"(R), "n"(R + 3), "n"(OFFSET)
                 : "memory");
}
template <int SLOT, int I_HI, int I_LO, int W>
__device__ __forceinline__ uint32_t ring_perm(uint32_t selector)
{
    constexpr int RH = kRingBase + 16 * SLOT + 4 * I_HI + W, RL = kRingBase + 16 * SLOT + 4 * I_LO + W;
    uint32_t x;
    asm volatile("v_perm_b32 %0, v[%1], v[%2], %3" : "=v"(x) : "n"(RH), "n"(RL), "s"(selector) : "memory");
    return x;
}
// The kernel's register count must cover the ring: one statement that names its last register.
__device__ __forceinline__ void ring_reserve() { asm volatile("" ::: "v255"); }

template <int N>
__device__ __forceinline__ void wait_loads_outstanding()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The four page ids of a tile, through the scalar cache.  Written as asm because the compiler
// would fetch them with vector loads here and wait for those with vmcnt(0).  The fetch is split
// from its wait: a tile's ids are requested one iteration before the tile's loads are issued,
// and the wait rides on the workgroup barrier in between.  One 16-byte scalar load per tile,
// unclamped: a tile that straddles the end of the entry picks up the next entry's ids (or the
// zeros the planner pads the list with), which are valid pages whose tokens are masked later;
// tiles past the end are requested but never loaded.
struct PageIds {
    i32x4 id;
};
__device__ __forceinline__ void page_ids_request(const int32_t *pages, int tile, PageIds &out)
{
    const int off = __builtin_amdgcn_readfirstlane(16 * tile);
    asm volatile("s_load_dwordx4 %0, %1, %2" : "=&s"(out.id) : "s"(pages), "s"(off) : "memory");
}
// The ids pass through the waiting asm as in/out operands, so nothing can use them earlier.
__device__ __forceinline__ void page_ids_wait(PageIds &p)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(p.id)::"memory");
}
__device__ __forceinline__ void lds_barrier_and_page_ids(PageIds &p)
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : "+s"(p.id)::"memory");
}

// v_max_f32 / v_max3_f32 as such (see compute_half).
__device__ __forceinline__ float max2(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

template <typename T, int ROW_WAVES>
__device__ __forceinline__ void tile_packed(const FwdArgs &a, const DevEntry &e, const UnitRec &up,
                                            int unit, int kvh, int tid, unsigned char *smem)
{
    using namespace pk;
    // Nothing is in flight here, but the compiler cannot tell: the tile functions are inlined
    // one after the other, and registers that another tile's loads were aimed at still count as
    // pending when this code is reached.  It would then guard their reuse by the (to it opaque)
    // asm loads below with waits that, at run time, drain this tile's own loads.  A wait it
    // understands clears that state.
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0), nothing else

    // tid: 0..511
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // 0..7
    // row group (rows 32 rg .. 32 rg + 31) and token half (tokens 32 th .. of a tile).  Four row
    // groups: the two halves of a group share a SIMD.  Two row groups: the four computing
    // wavefronts are 0..3, one per SIMD, and 4..7 only load.
    const int rg = ROW_WAVES == 4 ? (wave & 3) : (wave & 1);
    const int th = ROW_WAVES == 4 ? (wave >> 2) : ((wave >> 1) & 1);
    const int l32 = lane & 31;
    const int h = lane >> 5;
    const int G = a.G;
    const bool computes = ROW_WAVES == 4 || wave < 4;    // wavefront-uniform
    const int n_tiles = (e.n_pages + 3) >> 2;
    const int32_t *pages = a.page_ids + e.page_off;
    TraceMarks tm;

    // ---- loader role: odd wavefronts take V, even ones K; 256 threads each, 4 loads a tile ----
    // Every load instruction of a wavefront stays within one page, so its address is a scalar
    // base (pool, KV head, page, row block: scalar arithmetic on the page id) plus a per-lane
    // byte offset that never changes: no vector instruction is spent on addresses.
    const bool loads_v = (wave & 1) != 0;
    const int pw = wave >> 1;                           // 0..3 within the role
    const int r16 = lane & 15;                          // 16-byte piece of a 256-byte row
    //   K load i: token j + 8 (4 half + i) of the tile, j = sub_id, half = pw / 2:
    //             page 2 half + i / 2, row j + 8 (i % 2) of it
    //   V load i: position kappa = 4 half + i of group gamma = sub_id: page gamma / 2 = pw,
    //             row 8 half + 4 (gamma % 2) + i of it
    const int sub_id = loads_v ? 2 * pw + ((lane >> 4) & 1) : 4 * (pw & 1) + (lane >> 4);
    const int half = loads_v ? lane >> 5 : pw >> 1;
    const int id_a = loads_v ? pw : 2 * (pw >> 1);      // which of the tile's four pages: loads 0, 1
    const int id_b = loads_v ? pw : 2 * (pw >> 1) + 1;  //                                 loads 2, 3
    const uint32_t lane_row = loads_v ? 8 * half + 4 * (sub_id & 1) : sub_id;
    const uint32_t lane_off = 2u * (8u * r16 + lane_row * (uint32_t)a.stride_token);     // bytes
    const uint16_t *pool = (loads_v ? a.v_pool : a.k_pool) + (int64_t)kvh * a.stride_head;
    // One instruction stream for both roles: the role only selects addresses.
    const int64_t step1 = loads_v ? a.stride_token : 8 * a.stride_token;      // load 1 (and 3) vs 0 (2)
    const int64_t step2 = loads_v ? 2 * a.stride_token : 0;                   // load 2 vs 0
    auto issue_loads = [&](const PageIds &ids, auto slot) {
        constexpr int S = decltype(slot)::value;
        const int32_t page_a = id_a == 0 ? ids.id[0] : id_a == 1 ? ids.id[1] : id_a == 2 ? ids.id[2] : ids.id[3];
        const int32_t page_b = id_b == 0 ? ids.id[0] : id_b == 1 ? ids.id[1] : id_b == 2 ? ids.id[2] : ids.id[3];
        const uint16_t *base_a = pool + (int64_t)page_a * a.stride_page;
        const uint16_t *base_b = pool + (int64_t)page_b * a.stride_page + step2;
        ring_load<S, 0>(base_a, lane_off);
        ring_load<S, 1>(base_a + step1, lane_off);
        ring_load<S, 2>(base_b, lane_off);
        ring_load<S, 3>(base_b + step1, lane_off);
    };
    // LDS byte addresses of this lane's first K row and first V^T row in buffer 0
    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t k_dst = lds_base + 2u * ((sub_id + 32 * half) * kKsPitch + 8 * r16);
    auto stage_tile = [&](int tile, auto slot) {
        constexpr int S = decltype(slot)::value;        // tile % 2: ring slot and LDS buffer alike
        unsigned char *dst = smem + S * kBufBytes;
        uint16_t *vt = reinterpret_cast<uint16_t *>(dst + kKBytes);
        if (!loads_v) {
            // token sub_id + 8 (4 half + i) -> row pitch 272 bytes, eight rows per load
            ring_store_lds<S, 0, S * kBufBytes + 0 * 16 * kKsPitch>(k_dst);
            ring_store_lds<S, 1, S * kBufBytes + 1 * 16 * kKsPitch>(k_dst);
            ring_store_lds<S, 2, S * kBufBytes + 2 * 16 * kKsPitch>(k_dst);
            ring_store_lds<S, 3, S * kBufBytes + 3 * 16 * kKsPitch>(k_dst);
            return;
        }
        // 4x8 transpose of 16-bit elements: for element 8 r16 + el the four tokens go, as
        // 8 bytes, to row d' = 16 el + r16 at positions 8 gamma + 4 half ..
        const int tile_valid = e.kv_len - tile * kTileTokens;
        uint2 lo[4], hi[4];
        if (tile_valid < kTileTokens) {
            // the entry's last tile: rows past kv_len may hold anything (NaN included): zero
            // them so that their zero weights cannot poison the product
            u32x4 buf[4] = {ring_read<S, 0>(), ring_read<S, 1>(), ring_read<S, 2>(), ring_read<S, 3>()};
            const int t0 = 16 * (sub_id >> 1) + 8 * half + 4 * (sub_id & 1);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (t0 + i >= tile_valid) buf[i] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                lo[w].x = __builtin_amdgcn_perm(buf[1][w], buf[0][w], 0x05040100u);
                lo[w].y = __builtin_amdgcn_perm(buf[3][w], buf[2][w], 0x05040100u);
                hi[w].x = __builtin_amdgcn_perm(buf[1][w], buf[0][w], 0x07060302u);
                hi[w].y = __builtin_amdgcn_perm(buf[3][w], buf[2][w], 0x07060302u);
            }
        } else {
            const uint32_t sel_lo = 0x05040100u, sel_hi = 0x07060302u;
#define PAT_RING_TRANSPOSE(W)                              \
    lo[W].x = ring_perm<S, 1, 0, W>(sel_lo);               \
    lo[W].y = ring_perm<S, 3, 2, W>(sel_lo);               \
    hi[W].x = ring_perm<S, 1, 0, W>(sel_hi);               \
    hi[W].y = ring_perm<S, 3, 2, W>(sel_hi);
            PAT_RING_TRANSPOSE(0) PAT_RING_TRANSPOSE(1) PAT_RING_TRANSPOSE(2) PAT_RING_TRANSPOSE(3)
#undef PAT_RING_TRANSPOSE
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            *reinterpret_cast<uint2 *>(vt + (32 * w + r16) * kVtPitch + 8 * sub_id + 4 * half) = lo[w];
            *reinterpret_cast<uint2 *>(vt + (32 * w + 16 + r16) * kVtPitch + 8 * sub_id + 4 * half) = hi[w];
        }
    };

    // ---- start-up --------------------------------------------------------------------------------
    // The page ids of the first two tiles come with the unit record, so their loads depend on
    // nothing else.  The request id (for q), the epilogue's destinations and the ids of tile 2
    // are fetched in one further round trip; chained round trips would each queue behind the
    // loads the whole chip issues in the kernel's first microsecond.  Everything the compiler
    // loads itself is consumed before the first asm load is issued: its waits do not count asm
    // loads, and one placed later would drain them.
    const int my_row = rg * 32 + l32;                   // row within the entry's block
    const bool live = computes && my_row < e.n_rows;
    const int q_row = e.row_begin + (live ? my_row : 0);
    static_assert(kUnitPages == 8, "two tiles of page ids in the unit record");
    PageIds first[3];
    first[0].id = up.p0;
    first[1].id = up.p1;
    page_ids_request(pages, 2, first[2]);
    const int q_req = a.req_ids[e.req_off + q_row / G];
    // Where the epilogue will put the rows this lane writes (row = lane / 4 of each 16-row
    // pass): parked in LDS until then (the loop has no registers to spare).
    int *park = reinterpret_cast<int *>(smem + 2 * kBufBytes) + rg * 5 * 64 + lane;
    if (th == 0 && computes) {
        park[0] = a.req_slot[e.req_off + q_row / G];
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int blk_row = min(rg * 32 + 16 * pass + (lane >> 2), max(e.n_rows - 1, 0));
            const int pos = e.req_off + (e.row_begin + blk_row) / G;
            park[(1 + pass) * 64] = a.req_slot[pos];
            park[(3 + pass) * 64] = a.req_ids[pos];
        }
    }
    const uint16_t *qp =
        a.q + ((int64_t)q_req * a.Hq + (kvh * G + q_row % G)) * kHeadDim + 8 * h;
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(qp)::"memory");       // nothing of the above is left
    page_ids_wait(first[2]);

    // Q^T operands: row l32 of this row group, elements 16c + 8h .. +8 of chunk c.  Issued
    // before K and V, so when the compiler waits for them at their first use (with a count that
    // knows nothing of the asm loads) everything it over-waits for is older than tile 1.
    u32x4 qop[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const u32x4 v = load16(qp + 16 * c);
        qop[c] = live ? v : u32x4{0u, 0u, 0u, 0u};
    }
    using Slot0 = std::integral_constant<int, 0>;
    using Slot1 = std::integral_constant<int, 1>;
    ring_reserve();
    issue_loads(first[0], Slot0{});                     // tile t lives in ring slot t % 2
    if (1 < n_tiles) issue_loads(first[1], Slot1{});
    tm.mark(a, 0);

    const float sc = a.scale * 1.4426950408889634f;
    f32x16 acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // ---- this wavefront's 32 tokens of one tile -------------------------------------------------
    // Scale > 0 commutes with max, so the row maximum is taken on the raw scores.
    // The fences keep the compiler's scheduler from regrouping the phases (it would hoist the
    // operand reads and cluster the MFMAs, and run out of registers).
#define SB __builtin_amdgcn_sched_barrier(0)
    auto compute_half = [&](const uint16_t *ks, const uint16_t *vt, int valid) {
        u32x4 kop[8], pop[2];
        SB;
#pragma unroll
        for (int c = 0; c < 8; ++c)
            kop[c] = *reinterpret_cast<const u32x4 *>(ks + (32 * th + l32) * kKsPitch + 16 * c + 8 * h);
        f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        SB;
#pragma unroll
        for (int c = 0; c < 8; ++c) s = Mma<T>::mfma32(kop[c], qop[c], s);
        SB;
        // the V^T operands are fetched underneath the softmax (into the registers K has left)
        u32x4 vop[8];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int n = 0; n < 2; ++n)
                vop[2 * b + n] = *reinterpret_cast<const u32x4 *>(
                    vt + (32 * b + l32) * kVtPitch + 8 * (4 * th + 2 * n + h));
        SB;
        if (valid < 32) {                               // uniform: only the entry's last tile
            // lane holds tokens 8 (v / 4) + 4 h + v % 4 of the half
            const int lim = valid - 4 * h;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (!(8 * (v >> 2) + (v & 3) < lim)) s[v] = -INFINITY;
        }
        // The maxima are written as instructions: fmaxf() would first canonicalise every MFMA
        // result (one more instruction per value) and then pair them two by two.  No value here
        // is a NaN that needs quieting: the scores are finite or -inf.  The first maximum is left
        // to the compiler, and fenced: it knows how long after an MFMA its result may be read,
        // and it does not check that for the operands of an asm statement.
        float mx = fmaxf(s[0], s[1]);
        SB;
        mx = max3(max3(mx, s[2], s[3]), max3(s[4], s[5], s[6]), max3(s[7], s[8], s[9]));
        mx = max3(mx, max3(s[10], s[11], s[12]), max3(s[13], s[14], s[15]));
        {
            // the other half of the row sits in lane +-32: one VALU lane swap instead of a trip
            // through the LDS crossbar, which would sit on the critical path between the two
            // products.  After the swap one of the two registers holds the lane's own value and
            // the other its partner's, whichever half the lane is in.  Written as asm because
            // the compiler's builtin for this instruction hands back its first result twice;
            // the idle cycles before and after are the ones the compiler puts around it.
            float other = mx;
            asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(mx), "+v"(other));
            mx = max2(mx, other);
        }
        const float m_new = max2(m_run, mx * sc);       // finite: the half has a valid token
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], sc, -m_new));
        float ps[4];                                    // four short chains instead of one long one
#pragma unroll
        for (int v = 0; v < 4; ++v) ps[v] = (s[v] + s[v + 4]) + (s[v + 8] + s[v + 12]);
        l_run = l_run * corr + ((ps[0] + ps[1]) + (ps[2] + ps[3]));
        m_run = m_new;
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                pop[n][u] = Mma<T>::pack2(s[8 * n + 2 * u], s[8 * n + 2 * u + 1]);
        // the accumulator only needs rescaling when some row's maximum moved, which becomes
        // rare after the first tiles (uniform branch)
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(corr != 1.f) != 0, 0)) {
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[b] *= corr;
        }
        SB;
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[b] = Mma<T>::mfma32(vop[2 * b + n], pop[n], acc[b]);
        SB;
    };
#undef SB
    auto compute_tile = [&](int t) {
        const unsigned char *src = smem + (t & 1) * kBufBytes;
        const uint16_t *ks = reinterpret_cast<const uint16_t *>(src);
        const uint16_t *vt = reinterpret_cast<const uint16_t *>(src + kKBytes);
        const int valid = e.kv_len - t * kTileTokens - 32 * th;    // of this wavefront's half
        // A half past kv_len holds nothing: skipped, its state stays as it is.
        if (computes && valid > 0) compute_half(ks, vt, valid);
    };

    // ---- main loop ----------------------------------------------------------------------------
    // Iteration t computes tile t from buffer t % 2, then stores tile t + 1 (landed meanwhile)
    // to the other buffer and refills its ring slot with tile t + 3.  Unrolled by two so that
    // the ring slots are compile-time constants.
    PageIds ids = first[2];                             // ids of the next tile to be issued
    wait_loads_outstanding<4>();                        // q and tile 0 have landed (tile 1 may not have)
    if (!(1 < n_tiles)) wait_loads_outstanding<0>();
#pragma unroll
    for (int c = 0; c < 8; ++c) asm volatile("" : "+v"(qop[c]));     // q is in: no wait for it later
    tm.mark(a, 3);
    stage_tile(0, Slot0{});
    if (2 < n_tiles) issue_loads(ids, Slot0{});
    page_ids_request(pages, 3, ids);
    lds_barrier_and_page_ids(ids);                      // (A) tile 0 staged
    // The two wavefronts of a SIMD take the halves of an iteration in opposite order: one
    // computes while the other moves the next tile into LDS, then they swap.  Started together
    // after each barrier they would otherwise run the same phase at the same time and queue for
    // the same pipe (LDS reads, MFMA, exponentials) instead of filling each other's gaps.
    auto step = [&](int t, auto slot) {                 // slot = ring slot of tile t + 1
        if (th == 0) compute_tile(t);
        if (t + 1 < n_tiles) {                          // every condition here is uniform
            if (t + 2 < n_tiles) wait_loads_outstanding<4>();       // t + 1 landed, t + 2 in flight
            else wait_loads_outstanding<0>();
            stage_tile(t + 1, slot);
            if (t + 3 < n_tiles) issue_loads(ids, slot);
        }
        if (th != 0) compute_tile(t);
        if (t == 0) tm.mark(a, 1);
        page_ids_request(pages, t + 4, ids);
        lds_barrier_and_page_ids(ids);                  // (B) one per tile
    };
    for (int t = 0; t < n_tiles; t += 2) {
        step(t, Slot1{});
        if (t + 1 < n_tiles) step(t + 1, Slot0{});
    }
    tm.mark(a, 2);
    tm.flush(a, unit);

    // ---- combine the two token halves of each row group ------------------------------------------
    // (the last (B) barrier has passed: the tile buffers are free)
    l_run += __shfl_xor(l_run, 32, 64);
    float *xchg = reinterpret_cast<float *>(smem + rg * kXchgBytes);
    if (th == 1 && computes) {
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<float4 *>(xchg + ((4 * b + j) * 64 + lane) * 4) =
                    make_float4(acc[b][4 * j], acc[b][4 * j + 1], acc[b][4 * j + 2], acc[b][4 * j + 3]);
        xchg[64 * 64 + lane] = m_run;
        xchg[64 * 64 + 64 + lane] = l_run;
    }
    lds_barrier();
    if (th == 1 || !computes) {
        lds_barrier();                                  // matches the barrier below
        return;
    }
    {
        const float m1 = xchg[64 * 64 + lane], l1 = xchg[64 * 64 + 64 + lane];
        const float m = fmaxf(m_run, m1);               // finite: half 0 saw the first token
        const float w0 = __builtin_amdgcn_exp2f(m_run - m), w1 = __builtin_amdgcn_exp2f(m1 - m);
        l_run = l_run * w0 + l1 * w1;
        m_run = m;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 o = *reinterpret_cast<const float4 *>(xchg + ((4 * b + j) * 64 + lane) * 4);
                acc[b][4 * j] = acc[b][4 * j] * w0 + o.x * w1;
                acc[b][4 * j + 1] = acc[b][4 * j + 1] * w0 + o.y * w1;
                acc[b][4 * j + 2] = acc[b][4 * j + 2] * w0 + o.z * w1;
                acc[b][4 * j + 3] = acc[b][4 * j + 3] * w0 + o.w * w1;
            }
    }
    lds_barrier();                                      // the exchange area may be reused

    // ---- epilogue ------------------------------------------------------------------------
    // Partial rows go out straight from the accumulator registers: a lane holds runs of four
    // consecutive d' of its row, so a row is written as 16-byte stores in the tile's own head-dim
    // order (the merge kernel knows which slots are laid out this way).  Only rows that are
    // final results (requests with a single item) take the path through LDS that restores the
    // true order.
    const int my_slot = park[0];
    const int out_slot[2] = {park[64], park[128]}, out_req[2] = {park[192], park[256]};
    const float inv = 1.f / l_run;
    const float lse = (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
    if (live && my_slot >= 0) {
        const int head = kvh * G + (e.row_begin + my_row) % G;
        float *dst = a.part_o + ((int64_t)my_slot * a.Hq + head) * kHeadDim + 4 * h;
        if (a.fuse_mode) {                              // uniform: merged inside this launch
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    store16_agent(dst + 32 * b + 8 * j, acc[b][4 * j] * inv, acc[b][4 * j + 1] * inv,
                                  acc[b][4 * j + 2] * inv, acc[b][4 * j + 3] * inv);
            if (h == 0) store1_agent(a.part_lse + (int64_t)my_slot * a.Hq + head, lse);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    store16_stream(dst + 32 * b + 8 * j, acc[b][4 * j] * inv, acc[b][4 * j + 1] * inv,
                                   acc[b][4 * j + 2] * inv, acc[b][4 * j + 3] * inv);
            if (h == 0) a.part_lse[(int64_t)my_slot * a.Hq + head] = lse;
        }
    }
    if (__builtin_amdgcn_ballot_w64(live && my_slot < 0) == 0) return;      // uniform
    float *os = reinterpret_cast<float *>(smem) + rg * 16 * kOsPitch;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if ((l32 >> 4) == pass) {
            // acc[b][v] = O^T[d' = 32 b + 8 (v / 4) + 4 h + v % 4][row l32]
            // d' = 16 el + r  <->  d = 8 r + el
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int dp = 32 * b + 8 * (v >> 2) + 4 * h + (v & 3);
                    const int d = 8 * (dp & 15) + (dp >> 4);
                    os[(l32 & 15) * kOsPitch + d] = acc[b][v] * inv;
                }
        }
        // lse of the 16 rows of this pass lives in lanes 16 pass .. 16 pass + 15
        const float lse_r = __shfl(lse, 16 * pass + (lane >> 2), 64);
        __builtin_amdgcn_wave_barrier();               // LDS is in order within a wavefront
        // lane -> (row = lane / 4, 32 consecutive floats starting at 32 (lane % 4))
        const int rr = lane >> 2;
        const int blk_row = rg * 32 + 16 * pass + rr;
        if (blk_row < e.n_rows && out_slot[pass] < 0) {
            const int head = kvh * G + (e.row_begin + blk_row) % G;
            const int slot = out_slot[pass];
            const int req = out_req[pass];
            const float *src = os + rr * kOsPitch + 32 * (lane & 3);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float o[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) o[k] = src[8 * c + k];
                store_row_chunk<T>(a, slot, req, head, 32 * (lane & 3) + 8 * c, o, lse_r,
                                   (lane & 3) == 0 && c == 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace pat
