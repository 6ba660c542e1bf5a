// Forward tile TILE_VALU16: rows <= 16, VALU dot products (no matrix cores).
//
// A plain tile kept for small batches and for cross-checking the MFMA tiles on the GPU (the
// planner only picks it when asked to through force_tile).  The four wavefronts take the
// entry's tokens round-robin; a lane owns two of the 128 head-dim elements, so one K or V row
// is one coalesced 256-byte wavefront load.  Each wavefront keeps its own online-softmax
// state; the four states are combined through LDS at the end (sec. "Output Merge" applied
// inside the workgroup).
#pragma once
#include "pat_common.hip.h"

namespace pat {

// Runs on one 256-thread half of the workgroup, like the stream tile.
template <typename T>
__device__ __forceinline__ void tile_valu16(const FwdArgs &a, const DevEntry &e_in, int kvh,
                                            bool active, int tid, unsigned char *smem)
{
    constexpr int M = 16;
    DevEntry e = e_in;
    if (!active) {
        e.n_rows = 0;
        e.kv_len = 0;
    }
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int G = a.G;

    float2 qv[M];
#pragma unroll
    for (int r = 0; r < M; ++r) {
        qv[r] = make_float2(0.f, 0.f);
        if (r < e.n_rows) {
            const int row = e.row_begin + r;
            const int req = a.req_ids[e.req_off + row / G];
            const int head = kvh * G + row % G;
            const uint32_t w = *reinterpret_cast<const uint32_t *>(
                a.q + ((int64_t)req * a.Hq + head) * kHeadDim + 2 * lane);
            qv[r].x = Elem<T>::to_f32((uint16_t)(w & 0xffff)) * a.scale;
            qv[r].y = Elem<T>::to_f32((uint16_t)(w >> 16)) * a.scale;
        }
    }
    float m[M], l[M];
    float2 acc[M];
#pragma unroll
    for (int r = 0; r < M; ++r) {
        m[r] = -INFINITY;
        l[r] = 0.f;
        acc[r] = make_float2(0.f, 0.f);
    }

    for (int t = wave; t < e.kv_len; t += 4) {
        const int64_t page = a.page_ids[e.page_off + t / kPage];
        const int64_t off = page * a.stride_page + (int64_t)(t % kPage) * a.stride_token +
                            (int64_t)kvh * a.stride_head + 2 * lane;
        const uint32_t kw = *reinterpret_cast<const uint32_t *>(a.k_pool + off);
        const uint32_t vw = *reinterpret_cast<const uint32_t *>(a.v_pool + off);
        const float kx = Elem<T>::to_f32((uint16_t)(kw & 0xffff));
        const float ky = Elem<T>::to_f32((uint16_t)(kw >> 16));
        const float vx = Elem<T>::to_f32((uint16_t)(vw & 0xffff));
        const float vy = Elem<T>::to_f32((uint16_t)(vw >> 16));
#pragma unroll
        for (int r = 0; r < M; ++r) {
            if (r < e.n_rows) {                       // uniform across the wavefront
                const float s = wave_sum(qv[r].x * kx + qv[r].y * ky);
                const float mn = fmaxf(m[r], s);
                const float corr = __expf(m[r] - mn);       // exp(-inf) = 0 on the first token
                const float p = __expf(s - mn);
                l[r] = l[r] * corr + p;
                acc[r].x = acc[r].x * corr + p * vx;
                acc[r].y = acc[r].y * corr + p * vy;
                m[r] = mn;
            }
        }
    }

    // combine the four wavefront states: [4][16][128] floats, then [4][16] max and sum
    float *s_acc = reinterpret_cast<float *>(smem);
    float *s_m = s_acc + 4 * M * kHeadDim;
    float *s_l = s_m + 4 * M;
#pragma unroll
    for (int r = 0; r < M; ++r) {
        if (lane == 0) {
            s_m[wave * M + r] = m[r];
            s_l[wave * M + r] = l[r];
        }
        s_acc[(wave * M + r) * kHeadDim + 2 * lane] = acc[r].x;
        s_acc[(wave * M + r) * kHeadDim + 2 * lane + 1] = acc[r].y;
    }
    __syncthreads();
    const int r = tid >> 4;                           // thread -> (row, 8 head-dim elements)
    const int c0 = (tid & 15) * 8;
    if (r < e.n_rows) {
        const float mx = fmaxf(fmaxf(s_m[r], s_m[M + r]), fmaxf(s_m[2 * M + r], s_m[3 * M + r]));
        float w[4], lsum = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            w[k] = __expf(s_m[k * M + r] - mx);
            lsum += w[k] * s_l[k * M + r];
        }
        const float inv = 1.f / lsum;
        float o[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float x = 0.f;
#pragma unroll
            for (int k = 0; k < 4; ++k) x += w[k] * s_acc[(k * M + r) * kHeadDim + c0 + c];
            o[c] = x * inv;
        }
        const int row = e.row_begin + r;
        const int pos = e.req_off + row / G;
        store_row_chunk<T>(a, a.req_slot[pos], a.req_ids[pos], kvh * G + row % G, c0, o,
                           mx + __logf(lsum), (tid & 15) == 0);
    }
}

}  // namespace pat
