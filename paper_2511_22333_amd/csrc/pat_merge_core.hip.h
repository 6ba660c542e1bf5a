// One (request, q head) of the merge stage by ONE wavefront (sec. "Output Merge"): the two 32-lane
// halves take the even and the odd partials of the request's list and are added at the end.  Used
// by the merge kernel's "lists" mapping and by the forward kernel where it merges a request itself.
#pragma once
#include "pat_common.hip.h"

namespace pat {

// A 32-lane half holds one output row in the accumulation order: lane j has d = 32 (j % 4) + 8 i +
// j / 4 in component i.  Hands lane t of the half the elements 4 t .. 4 t + 3 (already rounded to
// T) and stores them as one 8-byte piece, so the half writes its 256-byte row whole.  Every lane of
// the wavefront must call; only halves with `active` store.
template <typename T>
__device__ __forceinline__ void store_row_in_order(uint16_t *row, float4 v, int lane, bool active)
{
    const int t = lane & 31, i = (t & 7) >> 1;
    const uint32_t p0 = (uint32_t)Elem<T>::from_f32(v.x) | (uint32_t)Elem<T>::from_f32(v.y) << 16;
    const uint32_t p1 = (uint32_t)Elem<T>::from_f32(v.z) | (uint32_t)Elem<T>::from_f32(v.w) << 16;
    uint32_t e[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        // element d = 4 t + c lives in lane 4 (d % 8) + d / 32, component (d % 32) / 8 = i
        const int src = (lane & 32) + 4 * (4 * (t & 1) + c) + (t >> 3);
        const uint32_t q0 = __shfl(p0, src, 64), q1 = __shfl(p1, src, 64);
        const uint32_t q = (i & 2) ? q1 : q0;
        e[c] = (i & 1) ? q >> 16 : q & 0xffffu;
    }
    if (active) *reinterpret_cast<uint2 *>(row + 4 * t) = make_uint2(e[0] | e[1] << 16, e[2] | e[3] << 16);
}

// rec: the request's 128-byte merge record.  Every lane of the wavefront must call.  AGENT: the
// partials were written earlier in the SAME launch (at agent scope) and are read past the L2.
template <typename T, bool AGENT = false>
__device__ __forceinline__ void merge_head_lists(const MergeArgs &a, const int32_t *rec, int head, int lane)
{
    const int half = lane >> 5, j = lane & 31;
    const int req = rec[0], n_total = rec[1], s0 = rec[2];
    const int slot_inline = rec[4 + min(j, kMergeInline - 1)];  // fetched along with the header
    // lane's elements: d' = 4 j + i, i = 0..3, i.e. d = 32 (j % 4) + 8 i + j / 4
    const int d0 = 32 * (j & 3) + (j >> 2);
    float mx = -INFINITY, total = 0.f;                  // total, acc: this half's share
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c0 = 0; c0 < n_total; c0 += kMergeInline) {        // chunks of up to 28 partials
        const int n = min(kMergeInline, n_total - c0);
        int slot = 0;                                   // bit 30: partial in the d' order
        float l = -INFINITY;
        if (j < n) {                                    // the same list in both halves
            slot = c0 == 0 ? slot_inline : a.req_slot_ids[s0 + c0 + j];
            l = load1<AGENT>(a.part_lse + (int64_t)(slot & ~kPartialPermutedBit) * a.Hq + head);
        }
        for (int i0 = 0; i0 < n; i0 += 16) {            // partial i0 + 2 k + half, k = 0..7
            float4 o[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                o[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                const int idx = i0 + 2 * k + half;
                const int sraw = __shfl(slot, min(idx, 31), 64);        // (every lane takes part)
                if (idx >= n) continue;
                const float *row =
                    a.part_o + ((int64_t)(sraw & ~kPartialPermutedBit) * a.Hq + head) * kHeadDim;
                if (sraw & kPartialPermutedBit)
                    o[k] = load4<AGENT>(row + 4 * j);
                else
                    o[k] = make_float4(load1<AGENT>(row + d0), load1<AGENT>(row + d0 + 8), load1<AGENT>(row + d0 + 16),
                                       load1<AGENT>(row + d0 + 24));
            }
            // one maximum for both halves: over lanes i0 .. i0 + 15 of the list
            float cm = (j >= i0 && j < i0 + 16) ? l : -INFINITY;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
            cm = __shfl(cm, i0, 64);
            const float m_new = fmaxf(mx, cm);
            const float corr = __expf(mx - m_new);      // 0 on the first batch
            total *= corr;
            acc.x *= corr; acc.y *= corr; acc.z *= corr; acc.w *= corr;
            mx = m_new;
            const float w = __expf(l - mx);             // 0 for lanes without a partial
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int idx = i0 + 2 * k + half;
                const float wk = __shfl(w, min(idx, 31), 64);
                if (idx >= n) continue;
                total += wk;
                acc.x += wk * o[k].x; acc.y += wk * o[k].y;
                acc.z += wk * o[k].z; acc.w += wk * o[k].w;
            }
        }
    }
    // the other half's share (same maximum in both)
    total += __shfl_xor(total, 32, 64);
    acc.x += __shfl_xor(acc.x, 32, 64);
    acc.y += __shfl_xor(acc.y, 32, 64);
    acc.z += __shfl_xor(acc.z, 32, 64);
    acc.w += __shfl_xor(acc.w, 32, 64);
    const float inv = 1.f / total;                      // both halves hold the whole sums now
    store_row_in_order<T>(a.out + ((int64_t)req * a.Hq + head) * kHeadDim,
                          make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv), lane, half == 0);
    if (a.lse && lane == 0) a.lse[(int64_t)req * a.Hq + head] = mx + __logf(total);
}

}  // namespace pat
