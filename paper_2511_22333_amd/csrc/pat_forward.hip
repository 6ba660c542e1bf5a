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
#include "pat_tile_packed.cuh"
#include "pat_tile_stream16.cuh"
#include "pat_tile_valu16.cuh"
#include "pat_tile_wave16.cuh"

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

template <typename T>
__global__ __launch_bounds__(512, 2) __attribute__((amdgpu_num_vgpr(kVgprLimitAttr))) void forward_kernel(
    FwdArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kFwdSmemBytes];
    run_unit<T, false>(a, blockIdx.x, smem);
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
