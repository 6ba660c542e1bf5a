// Forward tile TILE_WAVE16: up to 16 query rows, KV tile n = 32 tokens, ONE wavefront per item.
//
// The short-KV member of the 16-row family (sec. "Multi-tile Kernel", "Deriving KV tile n": a
// small n for short KV).  TILE_STREAM16 puts four wavefronts on one (entry, KV head) and joins
// them at the end; for entries of a few hundred tokens the start-up (record, first K/V round
// trip) and the join are most of a workgroup's life and nothing is in flight meanwhile.  Here an
// item = (entry, KV head) belongs to a single wavefront, which walks ALL its 32-token stages and
// then goes straight on to the next item of its list: the planner hands every wavefront of a
// persistent workgroup a list of items, the eight wavefronts of a CU run independently (no
// barrier, no shared LDS), and at an item boundary the next item's q rows and first K/V stage are
// requested BEFORE the finished item's result is normalised and stored.  So a CU always has
// several streams in flight, and one item's start-up and epilogue hide behind the others.
//
// Data movement and the two products per stage are those of TILE_STREAM16 (K through a
// wavefront-private LDS slab, V transposed in registers, S^T = K Q^T and O^T += V^T P^T with
// v_mfma_f32_16x16x32).  The epilogue needs no LDS: a lane holds 32 consecutive head-dim elements
// of its row.
#pragma once
#include "pat_common.hip.h"

namespace pat {

namespace w16 {
constexpr int kKsRow = 136;                 // halves per staged K row: 128 + 8 pad (272 bytes)
constexpr int kStageTokens = 32;            // tokens per stage (two pages)
constexpr int kSlabBytes = kStageTokens * kKsRow * 2;         // 8704 per wavefront
static_assert(8 * kSlabBytes <= kFwdSmemBytes, "LDS budget");
}  // namespace w16

// One wavefront: items [begin, end) of a.wave_items, one after the other.  `smem`: this
// wavefront's slab.  `trace_base`: index of item 0's timeline record.
template <typename T>
__device__ __forceinline__ void wave_stream16(const FwdArgs &a, int begin, int end, int lane,
                                              unsigned char *smem, int trace_base)
{
    using namespace w16;
    const int l16 = lane & 15;               // MFMA index within the 16-wide dimension
    const int grp = lane >> 4;               // 0..3: contraction sub-range
    const int G = a.G;
    const float sc = a.scale * 1.4426950408889634f;     // scores in the log2 domain
    uint16_t *ks = reinterpret_cast<uint16_t *>(smem);
    // K loads: load i covers tokens 4i + grp, elements l16*8 .. +8
    const int64_t k_lane = (int64_t)grp * a.stride_token + l16 * 8;
    // V loads: tokens 4*grp + j of each page, elements l16*8 .. +8
    const int64_t v_lane = (int64_t)(4 * grp) * a.stride_token + l16 * 8;

    // An item record is 16 ints; lane l holds int l % 16 of it, fields are read with readlane.
    auto rec_load = [&](int k) {
        return reinterpret_cast<const int32_t *>(a.wave_items + k)[lane & 15];
    };
    struct Item {
        int req_off, n_req, page_off, n_pages, kv_len, row_begin, n_rows, kvh, req0, slot0, page0, page1;
    };
    auto rec_decode = [&](int v) {
        Item it;
        it.req_off = __builtin_amdgcn_readlane(v, 0);
        it.n_req = __builtin_amdgcn_readlane(v, 1);
        it.page_off = __builtin_amdgcn_readlane(v, 2);
        it.n_pages = __builtin_amdgcn_readlane(v, 3);
        it.kv_len = __builtin_amdgcn_readlane(v, 4);
        it.row_begin = __builtin_amdgcn_readlane(v, 5);
        it.n_rows = __builtin_amdgcn_readlane(v, 6);
        it.kvh = __builtin_amdgcn_readlane(v, 7);
        it.req0 = __builtin_amdgcn_readlane(v, 8);
        it.slot0 = __builtin_amdgcn_readlane(v, 9);
        it.page0 = __builtin_amdgcn_readlane(v, 10);
        it.page1 = __builtin_amdgcn_readlane(v, 11);
        return it;
    };

    u32x4 kbuf[8], vbuf[8];
    auto issue_loads = [&](int kvh, int page_a, int page_b) {
        const int64_t head_off = (int64_t)kvh * a.stride_head;
        const int64_t base_a = (int64_t)page_a * a.stride_page + head_off;
        const int64_t base_b = (int64_t)page_b * a.stride_page + head_off;
        const uint16_t *ka = a.k_pool + base_a + k_lane, *kb = a.k_pool + base_b + k_lane;
        const uint16_t *va = a.v_pool + base_a + v_lane, *vb = a.v_pool + base_b + v_lane;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kbuf[i] = load16_stream(ka + (int64_t)(4 * i) * a.stride_token);
            kbuf[4 + i] = load16_stream(kb + (int64_t)(4 * i) * a.stride_token);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            vbuf[j] = load16_stream(va + (int64_t)j * a.stride_token);
            vbuf[4 + j] = load16_stream(vb + (int64_t)j * a.stride_token);
        }
    };
    // Q^T operand of an item (lane holds row l16, elements c*32 + grp*8 .. +8 of chunk c) and
    // where its row's result goes (request id, partial slot or -1).
    struct RowDst { int req, slot; };
    auto load_q = [&](const Item &it, u32x4 (&qop)[4], RowDst &dst) {
        const bool live = l16 < it.n_rows;
        const int row = it.row_begin + (live ? l16 : 0);
        const int ri = row / G;                         // request position within the entry
        dst.req = it.req0;
        dst.slot = it.slot0;
        if (it.n_req > 1) {                             // uniform; rare for this tile
            dst.req = a.req_ids[it.req_off + ri];
            dst.slot = a.req_slot[it.req_off + ri];
        }
        const int head = it.kvh * G + row % G;
        const uint16_t *qp = a.q + ((int64_t)dst.req * a.Hq + head) * kHeadDim + grp * 8;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const u32x4 v = load16(qp + c * 32);
            qop[c] = live ? v : u32x4{0u, 0u, 0u, 0u};
        }
    };

    // ---- first item: nothing to hide behind -------------------------------------------------------
    Item cur = rec_decode(rec_load(begin));
    u32x4 qop[4];
    RowDst dst;
    load_q(cur, qop, dst);
    issue_loads(cur.kvh, cur.page0, cur.page1);
    int k = begin;
    int rec_next = k + 1 < end ? rec_load(k + 1) : 0;
    unsigned long long t_start = 0;
    if (a.trace) t_start = wall_clock64();

    for (;;) {
        const int n_stages = (cur.n_pages + 1) >> 1;
        const int32_t *pages = a.page_ids + cur.page_off;
        // page ids one stage ahead of the loads, which are one stage ahead of the products
        int next_pa = 0, next_pb = 0;
        if (1 < n_stages) {
            next_pa = pages[2];
            next_pb = pages[min(3, cur.n_pages - 1)];
        }
        f32x4 acc[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m_run = -INFINITY, l_run = 0.f;
        const bool have_next = k + 1 < end;
        Item nxt = cur;
        u32x4 qnext[4];
        RowDst dnext = dst;

        for (int stage = 0; stage < n_stages; ++stage) {
            // ---- K: registers -> wavefront-private LDS slab (row = token, 272-byte pitch) -----
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<u32x4 *>(ks + (4 * i + grp) * kKsRow + l16 * 8) = kbuf[i];
            // LDS executes one wavefront's instructions in order: the reads below see these writes
            __builtin_amdgcn_wave_barrier();
            u32x4 vcur[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) vcur[j] = vbuf[j];
            if (stage + 1 < n_stages) {
                issue_loads(cur.kvh, next_pa, next_pb);
                if (stage + 2 < n_stages) {
                    next_pa = pages[2 * (stage + 2)];
                    next_pb = pages[min(2 * (stage + 2) + 1, cur.n_pages - 1)];   // clamp: masked if absent
                }
            } else if (have_next) {
                // the item's last stage: the next item's q rows and first stage go out now, its
                // record after next is asked for
                nxt = rec_decode(rec_next);
                load_q(nxt, qnext, dnext);
                issue_loads(nxt.kvh, nxt.page0, nxt.page1);
                rec_next = k + 2 < end ? rec_load(k + 2) : 0;
            }

            // ---- S^T = K . Q^T for both pages ---------------------------------------------------
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const u32x4 k0 = *reinterpret_cast<const u32x4 *>(ks + l16 * kKsRow + c * 32 + grp * 8);
                const u32x4 k1 =
                    *reinterpret_cast<const u32x4 *>(ks + (16 + l16) * kKsRow + c * 32 + grp * 8);
                s0 = Mma<T>::mfma16(k0, qop[c], s0);
                s1 = Mma<T>::mfma16(k1, qop[c], s1);
            }
            // lane holds tokens grp*4 + v of page A (s0) and page B (s1) for query row l16
            const int tok0 = stage * kStageTokens + grp * 4;
            const int valid = cur.kv_len - tok0;        // tokens tok0 + v valid iff v < valid
            float p[8];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[v] = v < valid ? s0[v] * sc : -INFINITY;
                p[4 + v] = (16 + v) < valid ? s1[v] * sc : -INFINITY;
            }
            float mx = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])),
                             fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);       // finite: every stage has a valid token
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            float psum = 0.f;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                p[v] = __builtin_amdgcn_exp2f(p[v] - m_new);
                psum += p[v];
            }
            l_run = l_run * corr + psum;                // per-lane part of the row sum
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {     // uniform; rare after warm-up
#pragma unroll
                for (int b = 0; b < 8; ++b) acc[b] *= corr;
            }
            // P^T operand: contraction index k = grp*8 + {A tokens 4grp..+3, B tokens 4grp..+3}
            const u32x4 pop = {Mma<T>::pack2(p[0], p[1]), Mma<T>::pack2(p[2], p[3]),
                               Mma<T>::pack2(p[4], p[5]), Mma<T>::pack2(p[6], p[7])};

            // ---- V: zero rows past kv_len (their memory may hold anything), transpose, MFMA -----
            if (stage * kStageTokens + kStageTokens > cur.kv_len) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (!(j < valid)) vcur[j] = u32x4{0u, 0u, 0u, 0u};
                    if (!((16 + j) < valid)) vcur[4 + j] = u32x4{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                // elements 2w (low halves) and 2w+1 (high halves) of the lane's 8 head-dim elements
                u32x4 lo, hi;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    lo[u] = __builtin_amdgcn_perm(vcur[2 * u + 1][w], vcur[2 * u][w], 0x05040100u);
                    hi[u] = __builtin_amdgcn_perm(vcur[2 * u + 1][w], vcur[2 * u][w], 0x07060302u);
                }
                acc[2 * w] = Mma<T>::mfma16(lo, pop, acc[2 * w]);
                acc[2 * w + 1] = Mma<T>::mfma16(hi, pop, acc[2 * w + 1]);
            }
            __builtin_amdgcn_wave_barrier();      // slab reads of this stage stay above the next writes
        }

        // ---- the item's result: row l16, elements 32 grp + 8 v + b = acc[b][v] ----------------
        l_run += __shfl_xor(l_run, 16, 64);
        l_run += __shfl_xor(l_run, 32, 64);
        if (l16 < cur.n_rows) {
            const float inv = 1.f / l_run;
            const float lse = (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
            const int row = cur.row_begin + l16;
            const int head = cur.kvh * G + row % G;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float o[8];
#pragma unroll
                for (int b = 0; b < 8; ++b) o[b] = acc[b][v] * inv;
                store_row_chunk<T>(a, dst.slot, dst.req, head, 32 * grp + 8 * v, o, lse, grp == 0 && v == 0);
            }
        }
        if (a.trace && lane == 0) {
            unsigned long long *rec = a.trace + 8ull * (trace_base + k);
            const unsigned long long t_end = wall_clock64();
            rec[0] = t_start;
            rec[1] = t_end;
            rec[2] = ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |
                     (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);      // XCC_ID, HW_ID
            rec[3] = ((unsigned long long)TILE_WAVE16 << 32) | (unsigned)cur.kv_len;
            t_start = t_end;
        }
        if (!have_next) break;
        cur = nxt;
        dst = dnext;
#pragma unroll
        for (int c = 0; c < 4; ++c) qop[c] = qnext[c];
        ++k;
    }
}

}  // namespace pat
