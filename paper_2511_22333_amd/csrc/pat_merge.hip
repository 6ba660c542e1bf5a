// Merge stage (sec. "Output Merge"): per (request, q head), combine the request's fp32
// partials by log-sum-exp:  L = logsumexp_i LSE_i,  out = sum_i exp(LSE_i - L) O_i.
//
// A lane owns four head-dim elements, so a partial row is one 16-byte load per lane of a
// 32-lane half.  Only requests with more than one partial are listed: the others were written
// in final form by the forward kernel.  Two mappings of the work to wavefronts:
//   pairs: one wavefront per (request, pair of q heads), a half per head -- for requests with
//          few partials (the merge is then a matter of throughput: fewer wavefronts);
//   lists: one wavefront per (request, q head), the halves take the even and the odd partials of
//          the list and are added at the end -- for long lists (one-round batches under a long
//          shared prefix), where the chain of round trips per wavefront is what counts.
// The kernel is a chain of dependent memory round trips, so it keeps the chain short: a request's
// record holds its id, the number of its partials and the first 28 slot ids, lane i fetches
// slot id i from it, then the LSEs and up to eight partial rows per half are requested together
// before any of them is used: two round trips before the arithmetic.
//
// The accumulation runs in the packed tiles' head-dim order d' = 16 (d % 8) + d / 8 (most
// partials of a request under a shared prefix come from packed tiles and are laid out that
// way); partials in the true order are gathered with four 4-byte loads, and the result is
// brought back to the true order through lane shuffles, so that a row leaves as whole 8-byte pieces.
#include "pat_merge_core.hip.h"

namespace pat {

template <typename T>
__global__ __launch_bounds__(256) void merge_kernel_pairs(MergeArgs a)
{
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5, j = lane & 31;
    const int pairs = (a.Hq + 1) >> 1;
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= a.n_merge * pairs) return;              // whole wavefront leaves together
    const int32_t *rec = a.merge_rec + (int64_t)(unit / pairs) * kMergeRecInts;
    const int req = rec[0], n_total = rec[1], s0 = rec[2];
    const int slot_inline = rec[4 + min(j, kMergeInline - 1)];  // fetched along with the header
    const int head = min(2 * (unit % pairs) + half, a.Hq - 1);
    const bool owner = 2 * (unit % pairs) + half < a.Hq;   // odd Hq: the last half is a duplicate
    // lane's elements: d' = 4 j + i, i = 0..3, i.e. d = 32 (j % 4) + 8 i + j / 4
    const int d0 = 32 * (j & 3) + (j >> 2);
    float mx = -INFINITY, total = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c0 = 0; c0 < n_total; c0 += kMergeInline) {        // chunks of up to 28 partials
        const int n = min(kMergeInline, n_total - c0);
        int slot = 0;                                   // bit 30: partial in the d' order
        float l = -INFINITY;
        if (j < n) {
            slot = c0 == 0 ? slot_inline : a.req_slot_ids[s0 + c0 + j];
            l = a.part_lse[(int64_t)(slot & ~kPartialPermutedBit) * a.Hq + head];
        }
        for (int i0 = 0; i0 < n; i0 += 8) {
            float4 o[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                o[k] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i0 + k >= n) continue;              // uniform
                const int sraw = __shfl(slot, i0 + k, 64);      // same list in both halves
                const float *row =
                    a.part_o + ((int64_t)(sraw & ~kPartialPermutedBit) * a.Hq + head) * kHeadDim;
                if (sraw & kPartialPermutedBit)         // uniform
                    o[k] = *reinterpret_cast<const float4 *>(row + 4 * j);
                else
                    o[k] = make_float4(row[d0], row[d0 + 8], row[d0 + 16], row[d0 + 24]);
            }
            float cm = (j >= i0 && j < i0 + 8) ? l : -INFINITY;
#pragma unroll
            for (int off = 4; off >= 1; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
            cm = __shfl(cm, 32 * half + i0, 64);        // max over this half's lanes i0 .. i0 + 7
            const float m_new = fmaxf(mx, cm);
            const float corr = __expf(mx - m_new);      // 0 on the first batch
            total *= corr;
            acc.x *= corr; acc.y *= corr; acc.z *= corr; acc.w *= corr;
            mx = m_new;
            const float w = __expf(l - mx);             // 0 for lanes without a partial
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float wk = (i0 + k < n) ? __shfl(w, 32 * half + i0 + k, 64) : 0.f;
                total += wk;
                acc.x += wk * o[k].x; acc.y += wk * o[k].y;
                acc.z += wk * o[k].z; acc.w += wk * o[k].w;
            }
        }
    }
    const float inv = 1.f / total;
    store_row_in_order<T>(a.out + ((int64_t)req * a.Hq + head) * kHeadDim,
                          make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv), lane, owner);
    if (owner && a.lse && j == 0) a.lse[(int64_t)req * a.Hq + head] = mx + __logf(total);
}

template <typename T>
__global__ __launch_bounds__(256) void merge_kernel_lists(MergeArgs a)
{
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= a.n_merge * a.Hq) return;               // whole wavefront leaves together
    merge_head_lists<T>(a, a.merge_rec + (int64_t)(unit / a.Hq) * kMergeRecInts, unit % a.Hq,
                        threadIdx.x & 63);
}

hipError_t launch_merge(int dtype, const MergeArgs &a, hipStream_t s)
{
    if (a.n_merge == 0) return hipSuccess;
    const int units = a.n_merge * (a.long_lists ? a.Hq : (a.Hq + 1) / 2);
    dim3 grid((unsigned)((units + 3) / 4)), block(256);
    MergeArgs args = a;
    void *params[] = {&args};
    const void *fn;
    if (a.long_lists)
        fn = dtype == PAT_F16 ? (const void *)merge_kernel_lists<F16> : (const void *)merge_kernel_lists<BF16>;
    else
        fn = dtype == PAT_F16 ? (const void *)merge_kernel_pairs<F16> : (const void *)merge_kernel_pairs<BF16>;
    return hipLaunchKernel(fn, grid, block, params, 0, s);
}

}  // namespace pat
