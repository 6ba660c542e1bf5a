// The forward stage as ONE launch: every workgroup looks up its unit and runs the tile the
// planner chose for it.
//
// The paper launches one kernel per (m, n) tile configuration on its own stream so that the
// configurations overlap (sec. "Multi Kernel Forward", "Multi-Stream Forward").  On this GPU
// the same effect comes from a single kernel whose workgroups branch (uniformly) on the
// unit's tile id: shared-prefix tiles and leaf streams fill the chip together, there is one
// launch latency instead of one per configuration, and no stream fork/join.
//
// Where a launch of many rounds ends in long 16-row units, those are not workgroups of their own:
// as many persistent workgroups as there are CUs take them from a queue (an atomic counter), which
// saves a workgroup launch per unit.
//
// Every workgroup has 512 threads and the CU to itself (8 wavefronts x 256 VGPRs is the whole
// register file).  Packed tiles run all eight wavefronts on one KV head (4 row groups x 2
// token halves); the 16-row tiles run two KV heads side by side, one per 256-thread half.
// The compiler allocates v0..v223 only: the packed tile keeps loads in flight in v224..v255.
#include "pat_merge_core.hip.h"
#include "pat_tile_packed.hip.h"
#include "pat_tile_stream16.hip.h"
#include "pat_tile_valu16.hip.h"
#include "pat_tile_wave16.hip.h"

namespace pat {

// One unit: the tile the planner chose for it.  LOOPED: called from the queue workers' loop; the
// thread index then goes through an opaque copy, so that what is derived from it is computed
// inside the loop instead of being kept in registers across every tile function (which spills).
template <typename T, bool LOOPED>
__device__ __forceinline__ void run_unit(const FwdArgs &a, int u, unsigned char *smem)
{
    int tx = threadIdx.x;
    if (LOOPED) asm volatile("" : "+v"(tx));
    unsigned long long t_start = 0;
    if (a.trace) t_start = wall_clock64();
    // The record goes into scalar registers in one round trip (see UnitRec).
    UnitRec ur;
    unit_fetch(a.units + u, ur);
    DevEntry ue;
    ue.req_off = ur.req_off();
    ue.n_req = ur.n_req();
    ue.page_off = ur.page_off();
    ue.n_pages = ur.n_pages();
    ue.kv_len = ur.kv_len();
    ue.row_begin = ur.row_begin();
    ue.n_rows = ur.n_rows();
    ue.tile = ur.tile();
    const int kvh0 = ur.kvh0(), n_heads = ur.n_heads();
    const int tile = ue.tile;
    if (tile >= TILE_PACKED64) {
        if (tile == TILE_PACKED128)
            tile_packed<T, 4>(a, ue, ur, u, kvh0, tx, smem);
        else
            tile_packed<T, 2>(a, ue, ur, u, kvh0, tx, smem);
    } else {
        const int half = __builtin_amdgcn_readfirstlane(tx >> 8);
        const bool active = half < n_heads;
        const int kvh = kvh0 + (active ? half : 0);
        unsigned char *hsmem = smem + half * kHalfSmemBytes;
        if (tile == TILE_STREAM16)
            tile_stream16<T>(a, ue, ur, u, kvh, active, tx & 255, hsmem);
        else
            tile_valu16<T>(a, ue, kvh, active, tx & 255, hsmem);
    }
    // Per-unit timeline (the analogue of the paper's per-SM CTA pipelines, sec. "Ablation
    // Study"): start and end on the 100 MHz constant clock, where it ran, what it was.
    if (a.trace && threadIdx.x == 0) {
        unsigned long long *rec = a.trace + 8ull * u;
        rec[0] = t_start;
        rec[1] = wall_clock64();
        rec[2] = ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |
                 (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);      // XCC_ID, HW_ID
        rec[3] = ((unsigned long long)ue.tile << 32) | (unsigned)ue.kv_len;
    }
}

// ---- merge inside the forward launch (sec. "Output Merge" without a second kernel) ---------------
// Every (request with several partials, KV head) is a task with a state word: arrivals so far and
// two flags.  A workgroup that has stored its unit's partials makes them visible (fence), then
// adds one arrival to the task of every (request, KV head) its unit holds rows of.
//   Tasks nobody waits for ("abandoned"; all tasks of launches of many rounds): the workgroup whose
//   arrival completes the task merges it there and then.  Nothing ever waits.
//   Launches of one round: workgroups that are done with their unit also claim tasks in order
//   and poll, a bounded number of times, until the task's arrivals are complete, then merge it --
//   so the merges of a batch under one long shared prefix, whose partials all arrive at the very end,
//   are spread over the whole chip instead of falling to the last packed workgroup of each head.  A
//   claimer that runs out of polls marks the task abandoned and leaves: the arrival that completes
//   it sees the mark and merges.  Both sides decide on one atomic word, so exactly one of them merges.
// The merger puts the word back to its initial value; the last workgroup out resets the claim counters.
template <typename T>
__device__ __forceinline__ void fused_merge_task(const FwdArgs &a, int task)
{
    MergeArgs m;
    m.merge_rec = a.merge_rec;
    m.req_slot_ids = a.req_slot_ids;
    m.part_o = a.part_o;
    m.part_lse = a.part_lse;
    m.out = a.out;
    m.lse = a.lse;
    m.n_merge = a.n_merge;
    m.Hq = a.Hq;
    m.long_lists = 1;
    const int midx = task / a.Hkv, g = task % a.Hkv;
    const int32_t *rec = a.merge_rec + (int64_t)midx * kMergeRecInts;
    int tx = threadIdx.x;
    asm volatile("" : "+v"(tx));
    for (int hh = __builtin_amdgcn_readfirstlane(tx >> 6); hh < a.G; hh += 8)
        merge_head_lists<T, true>(m, rec, g * a.G + hh, tx & 63);
}

template <typename T>
__device__ __forceinline__ void fused_merge(const FwdArgs &a, int u)
{
    __shared__ int s_ready[160];
    __shared__ int s_n, s_task, s_do;
    const int init = a.fuse_mode == 1 ? kFuseAbandoned : 0;
    int tx = threadIdx.x;
    asm volatile("" : "+v"(tx));
    // this thread's partials (agent-scope stores: written through) have been acknowledged
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0)
    if (tx == 0) s_n = 0;
    __syncthreads();
    {
        const DevUnit *up = a.units + u;
        const int G = a.G;
        const int first = up->e.row_begin / G, last = (up->e.row_begin + up->e.n_rows - 1) / G;
        const int nh = up->n_heads;
        if (tx < (last - first + 1) * nh) {
            const int midx = a.req_midx[up->e.req_off + first + tx / nh];
            if (midx >= 0) {
                const int task = midx * a.Hkv + up->kvh0 + tx % nh;
                const int old = atomicAdd(a.merge_state + task, 1);
                if ((old & kFuseCountMask) + 1 == a.merge_rec[midx * kMergeRecInts + 3] && (old & kFuseAbandoned))
                    s_ready[atomicAdd(&s_n, 1)] = task;
            }
        }
    }
    __syncthreads();
    const int n = s_n;
    if (n > 0) {                                        // uniform
        for (int i = 0; i < n; ++i) fused_merge_task<T>(a, s_ready[i]);
        if (tx < n) a.merge_state[s_ready[tx]] = init;
    }
    if (a.fuse_mode != 2) return;
    const int n_tasks = a.n_merge * a.Hkv;
    for (;;) {
        if (tx == 0) {
            const int t = atomicAdd(a.queue_ctr, 1);
            int take = 0;
            if (t < n_tasks) {
                const int expected = a.merge_rec[(t / a.Hkv) * kMergeRecInts + 3];
                int cnt = atomicOr(a.merge_state + t, kFuseClaimed) & kFuseCountMask;
                for (int it = 0; cnt != expected && it < a.spin_limit; ++it) {
                    __builtin_amdgcn_s_sleep(32);
                    cnt = __hip_atomic_load(a.merge_state + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) &
                          kFuseCountMask;
                }
                if (cnt == expected)
                    take = 1;
                else
                    take = (atomicOr(a.merge_state + t, kFuseAbandoned) & kFuseCountMask) == expected;
            }
            s_task = t;
            s_do = take;
        }
        __syncthreads();
        const int t = s_task, take = s_do;
        __syncthreads();                                // s_task may be written again
        if (t >= n_tasks) break;
        if (take) {
            fused_merge_task<T>(a, t);
            if (tx == 0) a.merge_state[t] = init;
        }
    }
    if (tx == 0) {
        if (atomicAdd(a.queue_ctr + 1, 1) == (int)gridDim.x - 1) {
            a.queue_ctr[0] = 0;
            a.queue_ctr[1] = 0;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(kVgprLimitAttr))) void forward_kernel(
    FwdArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kFwdSmemBytes];
    run_unit<T, false>(a, blockIdx.x, smem);
    if (a.fuse_mode) fused_merge<T>(a, blockIdx.x);
}

// The same with a queue: workgroups below queue_begin run their own unit, the others are
// workers that take the next queued unit until none is left.  One thread draws the index,
// everybody reads it behind a barrier; the loop ends for every wavefront at the same draw.
// (Drawing one unit ahead would hide the atomic's round trip, but a worker that sits on a drawn
// unit while others have run dry costs more at the end of the launch than the round trips do:
// measured.)  The last worker to leave puts both counters back to zero for the next launch.
template <typename T>
__global__ __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(kVgprLimitAttr))) void forward_queue_kernel(
    FwdArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kFwdSmemBytes];
    __shared__ int next_unit;
    const int wg = blockIdx.x;
    const bool worker = wg >= a.queue_begin;            // uniform
    int u = wg;
    for (;;) {
        if (worker) {
            if (threadIdx.x == 0) next_unit = a.queue_begin + atomicAdd(a.queue_ctr, 1);
            __syncthreads();
            u = __builtin_amdgcn_readfirstlane(next_unit);
            __syncthreads();                            // next_unit may be written again
            if (u >= a.n_units) break;
        }
        run_unit<T, true>(a, u, smem);
        if (!worker) return;
        __syncthreads();                                // the tile's LDS is free again
    }
    if (threadIdx.x == 0) {
        __threadfence();
        if (atomicAdd(a.queue_ctr + 1, 1) == a.queue_workers - 1) {
            a.queue_ctr[0] = 0;
            a.queue_ctr[1] = 0;
        }
    }
}

// The 16-row tiles of a two-kernel launch (the paper's multi-stream forward, sec. "Multi-Stream
// Forward": kernels of different tile configurations side by side on streams of their own).
// A workgroup is 256 threads on ONE KV head with half a CU's registers, so two of them share a CU
// and are scheduled independently: while one waits for its unit record, its first K/V stage or
// its epilogue's stores, the other one streams.  (As halves of one 512-thread workgroup the two
// heads start, wait and end together, and nothing is in flight during those phases.)
template <typename T>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void forward_stream_kernel(
    FwdArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kHalfSmemBytes];
    const int u = a.unit_base + blockIdx.x;
    unsigned long long t_start = 0;
    if (a.trace) t_start = wall_clock64();
    UnitRec ur;
    unit_fetch(a.units + u, ur);
    DevEntry ue;
    ue.req_off = ur.req_off();
    ue.n_req = ur.n_req();
    ue.page_off = ur.page_off();
    ue.n_pages = ur.n_pages();
    ue.kv_len = ur.kv_len();
    ue.row_begin = ur.row_begin();
    ue.n_rows = ur.n_rows();
    ue.tile = ur.tile();
    if (ue.tile == TILE_STREAM16)
        tile_stream16<T>(a, ue, ur, u, ur.kvh0(), true, threadIdx.x, smem);
    else
        tile_valu16<T>(a, ue, ur.kvh0(), true, threadIdx.x, smem);
    if (a.trace && threadIdx.x == 0) {
        unsigned long long *rec = a.trace + 8ull * u;
        rec[0] = t_start;
        rec[1] = wall_clock64();
        rec[2] = ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |
                 (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);      // XCC_ID, HW_ID
        rec[3] = ((unsigned long long)ue.tile << 32) | (unsigned)ue.kv_len;
    }
}

hipError_t launch_forward_stream(int dtype, const FwdArgs &a, int n_workgroups, hipStream_t s)
{
    if (n_workgroups == 0) return hipSuccess;
    FwdArgs args = a;
    void *params[] = {&args};
    const void *fn = dtype == PAT_F16 ? (const void *)forward_stream_kernel<F16>
                                      : (const void *)forward_stream_kernel<BF16>;
    return hipLaunchKernel(fn, dim3((unsigned)n_workgroups), dim3(256), params, 0, s);
}

// Launches that hold wavefront items (TILE_WAVE16): as many persistent workgroups as the planner
// made lists for.  A workgroup first runs its workgroup-level units (packed tiles, long 16-row
// streams) one after the other, then its eight wavefronts part ways, each walking its own list of
// items; nothing waits for anything: the schedule is static.
template <typename T>
__global__ __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(kVgprLimitAttr))) void forward_worker_kernel(
    FwdArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kFwdSmemBytes];
    const int32_t *wrec = reinterpret_cast<const int32_t *>(a.workers + blockIdx.x);
    const int unit_begin = __builtin_amdgcn_readfirstlane(wrec[0]);
    const int unit_end = __builtin_amdgcn_readfirstlane(wrec[1]);
    for (int u = unit_begin; u < unit_end; ++u) {
        run_unit<T, true>(a, u, smem);
        __syncthreads();                                // the tile's LDS is free again
    }
    int tx = threadIdx.x;
    asm volatile("" : "+v"(tx));
    const int wave = __builtin_amdgcn_readfirstlane(tx >> 6);
    const int begin = __builtin_amdgcn_readfirstlane(wrec[2 + wave]);
    const int end = __builtin_amdgcn_readfirstlane(wrec[3 + wave]);
    if (begin < end)
        wave_stream16<T>(a, begin, end, tx & 63, smem + wave * w16::kSlabBytes, a.n_units);
}

hipError_t launch_forward(int dtype, const FwdArgs &a, int n_workgroups, hipStream_t s)
{
    if (n_workgroups == 0) return hipSuccess;
    dim3 grid((unsigned)n_workgroups), block(512);
    FwdArgs args = a;
    void *params[] = {&args};
    const void *fn;
    if (a.workers)
        fn = dtype == PAT_F16 ? (const void *)forward_worker_kernel<F16> : (const void *)forward_worker_kernel<BF16>;
    else if (a.queue_workers > 0)
        fn = dtype == PAT_F16 ? (const void *)forward_queue_kernel<F16> : (const void *)forward_queue_kernel<BF16>;
    else
        fn = dtype == PAT_F16 ? (const void *)forward_kernel<F16> : (const void *)forward_kernel<BF16>;
    // the launch's own status: hipGetLastError() could hand back an unrelated earlier failure
    return hipLaunchKernel(fn, grid, block, params, 0, s);
}

}  // namespace pat
