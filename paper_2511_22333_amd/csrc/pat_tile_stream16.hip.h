// Forward tile TILE_STREAM16: up to 16 query rows, MFMA, four independent wavefront streams.
//
// Used for leaves and small groups (rows = requests x GQA group <= 16), where the work is a
// pure HBM stream: a few flops per KV byte.  The workgroup's four wavefronts take 32-token
// stages (two pages) of the entry round-robin and never synchronise inside the loop.  Each
// wavefront keeps its own online-softmax state (sec. "Multi-tile Kernel": tiled pipeline with
// the next tile prefetched while the current one is computed); the four states are merged
// through LDS at the end (sec. "Output Merge" applied inside the workgroup) and one fp32
// partial or the final output is written.
//
// Data movement per stage and wavefront (16 KB: K and V of 32 tokens of one KV head):
//   K : 8 coalesced 16-byte loads per lane (16 lanes cover one 256-byte token row), staged
//       through a wavefront-private LDS slab to reach the MFMA operand layout
//       (lane = token, 8 consecutive head-dim elements per 32-wide contraction chunk).
//   V : 8 coalesced 16-byte loads per lane of the SAME 8 head-dim elements for the 8 tokens
//       the lane contracts over; an in-register 8x8 16-bit transpose (v_perm) yields the
//       operand (lane = head-dim element, 8 tokens).  No LDS traffic for V.
// Matrix products (v_mfma_f32_16x16x32, fp32 accumulate):
//   S^T[token][row] = K . Q^T      4 MFMAs per page, contraction over d = 128
//   O^T[d][row]    += V^T . P^T    8 MFMAs per stage, contraction over the 32 tokens
// In S^T a lane holds 4 tokens of ONE query row, so the running max needs two cross-lane
// steps and P goes from the accumulator registers straight into the next MFMA's operand.
#pragma once
#include "pat_common.hip.h"

namespace pat {

namespace s16 {
constexpr int kKsRow = 136;                 // halves per staged K row: 128 + 8 pad (272 bytes)
constexpr int kStageTokens = 32;            // tokens per wavefront stage (two pages)
constexpr int kOsRow = 132;                 // floats per row of the final merge buffer
constexpr int kSlabBytes = 4 * kStageTokens * kKsRow * 2;     // 34816
static_assert(kSlabBytes + 512 <= kHalfSmemBytes, "LDS budget");
static_assert(4 * 16 * kOsRow * 4 <= kSlabBytes, "merge buffer aliases the slabs");
}  // namespace s16

// Runs on one 256-thread half of the workgroup (`tid` = thread index within the half, `smem` =
// the half's LDS).  Both halves execute the same barriers: an idle half (active == false) walks
// through with nothing to load or store.
template <typename T>
__device__ __forceinline__ void tile_stream16(const FwdArgs &a, const DevEntry &e_in,
                                              const UnitRec &up, int unit, int kvh, bool active, int tid,
                                              unsigned char *smem)
{
    using namespace s16;
    float *s_m = reinterpret_cast<float *>(smem + kSlabBytes);       // [4][16]
    float *s_l = s_m + 64;                                           // [4][16]

    DevEntry e = e_in;
    if (!active) {
        e.n_rows = 0;
        e.n_pages = 0;
        e.kv_len = 0;
    }
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15;               // MFMA index within the 16-wide dimension
    const int grp = lane >> 4;               // 0..3: contraction sub-range
    const int G = a.G;

    const float sc = a.scale * 1.4426950408889634f;     // scores in the log2 domain
    f32x4 acc[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    const int n_stages = (e.n_pages + 1) >> 1;
    const int32_t *pages = a.page_ids + e.page_off;
    const int64_t head_off = (int64_t)kvh * a.stride_head;
    // K loads: load i covers tokens 4i + grp, elements l16*8 .. +8
    const int64_t k_lane = (int64_t)grp * a.stride_token + l16 * 8;
    // V loads: tokens 4*grp + j of each page, elements l16*8 .. +8
    const int64_t v_lane = (int64_t)(4 * grp) * a.stride_token + l16 * 8;
    uint16_t *ks = reinterpret_cast<uint16_t *>(smem) + wave * (kStageTokens * kKsRow);

    u32x4 kbuf[8], vbuf[8];
    auto issue_loads = [&](int stage, int page_a, int page_b) {
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

    // Start-up: the first stage's page ids (stage = wavefront, pages 2 wave and 2 wave + 1) and the
    // request ids of up to four requests come with the unit record, so the q rows and the first
    // K and V loads go out as soon as it is there.  Every dependent fetch here would cost a
    // round trip through a memory system that the whole chip is loading.
    TraceMarks tm;
    int stage = wave;
    const bool has_work = stage < n_stages;
    static_assert(kUnitPages == 8 && kUnitReqs == 4, "selects below");
    const int first_pa = wave == 0 ? up.page(0) : wave == 1 ? up.page(2)
                       : wave == 2 ? up.page(4) : up.page(6);
    const int first_pb = wave == 0 ? up.page(1) : wave == 1 ? up.page(3)
                       : wave == 2 ? up.page(5) : up.page(7);
    // ---- Q^T operand: lane holds row l16, elements c*32 + grp*8 .. +8 of chunk c ------------
    u32x4 qop[4];
    {
        const bool live = l16 < e.n_rows;
        const int row = e.row_begin + (live ? l16 : 0);
        const int ri = row / G;                         // request position within the entry
        int req = ri == 0 ? up.req(0) : ri == 1 ? up.req(1)
                : ri == 2 ? up.req(2) : up.req(3);
        if (e.n_req > kUnitReqs) req = a.req_ids[e.req_off + ri];          // uniform
        const int head = kvh * G + row % G;
        const uint16_t *qp = a.q + ((int64_t)req * a.Hq + head) * kHeadDim + grp * 8;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            u32x4 v = load16(qp + c * 32);
            qop[c] = live ? v : u32x4{0u, 0u, 0u, 0u};
        }
    }

    // Where the epilogue will put the row this thread writes: fetched now, alongside q (at the end
    // it would be one more round trip before the first store).
    const int out_r = tid >> 4;
    const int out_row = e.row_begin + (out_r < e.n_rows ? out_r : 0);
    const int out_pos = e.req_off + out_row / G;
    int out_slot = 0, out_req = 0;
    if (e.n_rows > 0) {                                 // uniform: an idle half has no entry
        out_slot = a.req_slot[out_pos];
        out_req = a.req_ids[out_pos];
    }

    if (has_work) issue_loads(stage, first_pa, first_pb);
    tm.mark(a, 3);
    // ids of the stage after that: always fetched one stage ahead, so that only the K/V loads
    // themselves are a round trip the loop has to wait for (asked for after the first loads have
    // gone out: nothing of the start-up waits for them)
    const bool has_second = stage + 4 < n_stages;
    int next_pa = has_second ? pages[2 * (stage + 4)] : 0;
    int next_pb = has_second ? pages[min(2 * (stage + 4) + 1, e.n_pages - 1)] : 0;

    for (; stage < n_stages; stage += 4) {
        // ---- K: registers -> wavefront-private LDS slab (row = token, 272-byte pitch) -------
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<u32x4 *>(ks + (4 * i + grp) * kKsRow + l16 * 8) = kbuf[i];
        // LDS executes one wavefront's instructions in order, so the reads below see these
        // writes without a barrier; the fence only pins the compiler's ordering.
        __builtin_amdgcn_wave_barrier();
        // V of this stage leaves the load registers through the transpose below; take a copy
        // so the next stage's loads can be issued right away.
        u32x4 vcur[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) vcur[j] = vbuf[j];
        const int next = stage + 4;
        if (next < n_stages) {
            issue_loads(next, next_pa, next_pb);
            const int after = next + 4;
            if (after < n_stages) {
                next_pa = pages[2 * after];
                next_pb = pages[min(2 * after + 1, e.n_pages - 1)];    // clamp: masked if absent
            }
        }
        if (stage == 0) tm.mark(a, 0);

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
        const int valid = e.kv_len - tok0;          // tokens tok0 + v valid iff v < valid
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
        if (stage * kStageTokens + kStageTokens > e.kv_len) {
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

    tm.mark(a, 2);
    tm.flush(a, unit);
    // ---- merge the four wavefront states ----------------------------------------------------
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    __syncthreads();                                  // every wavefront is done with its slab
    float *os = reinterpret_cast<float *>(smem);
    if (grp == 0) {
        s_m[wave * 16 + l16] = m_run;
        s_l[wave * 16 + l16] = l_run;
    }
    // acc[b][v] = O^T[d = 8*(4*grp + v) + b][row l16]
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            os[(wave * 16 + l16) * kOsRow + 8 * (4 * grp + v) + b] = acc[b][v];
    __syncthreads();
    const int r = tid >> 4;
    const int c0 = (tid & 15) * 8;
    if (r < e.n_rows) {
        const float mx = fmaxf(fmaxf(s_m[r], s_m[16 + r]), fmaxf(s_m[32 + r], s_m[48 + r]));
        float w[4], lsum = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            w[k] = __builtin_amdgcn_exp2f(s_m[k * 16 + r] - mx);
            lsum += w[k] * s_l[k * 16 + r];
        }
        const float inv = 1.f / lsum;
        float o[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float x = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) x += w[k] * os[(k * 16 + r) * kOsRow + c0 + c];
            o[c] = x * inv;
        }
        const float lse = (mx + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
        const int row = e.row_begin + r;            // r == out_r
        store_row_chunk<T>(a, out_slot, out_req, kvh * G + row % G, c0, o, lse, (tid & 15) == 0);
    }
}

}  // namespace pat
