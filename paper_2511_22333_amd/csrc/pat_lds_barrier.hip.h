// Workgroup barrier that orders LDS traffic only.
//
// __syncthreads() carries a workgroup-scope fence over all address spaces, which on this
// target makes the compiler wait for EVERY outstanding global load (s_waitcnt vmcnt(0)) before
// the barrier.  A tile pipeline that keeps global loads in flight across its barriers would
// lose all of its prefetch depth to that.  The tiles only exchange data through LDS, so the
// barrier here waits for the wavefront's LDS operations alone; registers that are still being
// loaded from global memory are waited for where they are first used.
#pragma once

namespace pat {

__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace pat
