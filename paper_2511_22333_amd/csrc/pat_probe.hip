// Measurement kernels of the benchmark and of the calibration runs (libpat_probe.so).  Not part of
// the attention path and not part of its ABI: plain memory kernels that say what the GPU's memory
// system can do, so that the attention kernels' numbers can be put against a measured ceiling
// (sec. "Multi-tile Kernel": the latency-versus-size microbenchmark whose flat part is the
// latency L and whose slope is the bandwidth B of the tile constraints).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}

// Streaming read: every wavefront owns one contiguous slice of the buffer and walks it in 1 KB rows
// (64 lanes x 16 bytes), sixteen rows in flight.
template <bool NT>
__global__ __launch_bounds__(512) void read_kernel(const u32x4 *base, size_t per_wave_vec, uint32_t *sink)
{
    constexpr int UNROLL = 16;
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const u32x4 *p = base + wave * per_wave_vec + (threadIdx.x & 63);
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = 0; i < per_wave_vec; i += 64 * UNROLL) {       // per_wave_vec % (64 * UNROLL) == 0
        u32x4 v[UNROLL];
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) v[k] = ld16<NT>(p + i + 64 * k);
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) acc ^= v[k];
    }
    // keeps the loads alive; the condition is practically never true
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}

// Latency versus request size: one wavefront-synchronous workgroup asks for `LOADS` 16-byte pieces
// per thread (256 * 16 * LOADS bytes, contiguous), waits until all of them are there, and does that
// `iters` times on fresh addresses.  Reports the mean time of one such request in nanoseconds.
template <int LOADS>
__global__ __launch_bounds__(256) void latency_kernel(const u32x4 *p, size_t n_vec, int iters, int seed,
                                                      float *ns_out, uint32_t *sink)
{
    const size_t chunk = (size_t)256 * LOADS;                     // vectors per request
    const size_t n_chunks = n_vec / chunk;
    u32x4 acc = {0u, 0u, 0u, 0u};
    // a different chunk per (iteration, workgroup), spread over the whole buffer
    // (`seed` moves every workgroup's walk: a second launch must not find the first one's lines cached)
    size_t c = ((size_t)blockIdx.x * 2654435761u + (size_t)seed * 40503u) % n_chunks;
    __syncthreads();
    const unsigned long long t0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        const u32x4 *q = p + c * chunk + threadIdx.x;
        u32x4 v[LOADS];
#pragma unroll
        for (int k = 0; k < LOADS; ++k) v[k] = __builtin_nontemporal_load(q + 256 * k);
#pragma unroll
        for (int k = 0; k < LOADS; ++k) acc ^= v[k];
        // the next request's address depends on this one's data: requests cannot overlap
        c = (c + 7919 * (size_t)gridDim.x + ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u)) % n_chunks;
        __syncthreads();
    }
    const unsigned long long t1 = wall_clock64();
    if (threadIdx.x == 0) ns_out[blockIdx.x] = (float)(t1 - t0) * 10.0f / (float)iters;   // 100 MHz clock
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}

}  // namespace

extern "C" {

// Reads device memory `buf` once with `workgroups` workgroups of 512 threads; every wavefront takes
// an equal contiguous slice (a multiple of 16 KB), so up to 16 KB * 8 * workgroups at the end of
// `bytes` stay unread: *bytes_read receives what was read.  nontemporal != 0: non-temporal loads.
// sink: 4 device bytes.  Returns 0 or a hipError_t; -1 for bad arguments.
int pat_probe_read(const void *buf, size_t bytes, int nontemporal, int workgroups, void *sink,
                   size_t *bytes_read, void *stream)
{
    if (!buf || !sink || !bytes_read || workgroups < 1) return -1;
    const size_t waves = (size_t)workgroups * 8;
    size_t per_wave_vec = bytes / 16 / waves;
    per_wave_vec -= per_wave_vec % (64 * 16);
    if (per_wave_vec == 0) return -1;
    *bytes_read = per_wave_vec * 16 * waves;
    const u32x4 *p = static_cast<const u32x4 *>(buf);
    uint32_t *s = static_cast<uint32_t *>(sink);
    void *params[] = {&p, &per_wave_vec, &s};
    const void *fn = nontemporal ? (const void *)read_kernel<true> : (const void *)read_kernel<false>;
    return (int)hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(512), params, 0,
                                static_cast<hipStream_t>(stream));
}

// `workgroups` workgroups each make `iters` dependent requests of 256 * 16 * loads_per_thread bytes
// (loads_per_thread in {1, 2, 4, 8, 16, 32}) from `buf` (`bytes` long, at least 64 requests), the
// walk through the buffer starting at a place that depends on `seed`;
// ns_out[workgroup] (device floats) receives the mean time per request.
int pat_probe_latency(const void *buf, size_t bytes, int loads_per_thread, int workgroups, int iters,
                      int seed, float *ns_out, void *sink, void *stream)
{
    if (!buf || !sink || !ns_out || workgroups < 1 || iters < 1) return -1;
    const u32x4 *p = static_cast<const u32x4 *>(buf);
    size_t n = bytes / 16;
    if (n < (size_t)64 * 256 * loads_per_thread) return -1;
    uint32_t *s = static_cast<uint32_t *>(sink);
    void *params[] = {&p, &n, &iters, &seed, &ns_out, &s};
    const void *fn;
    switch (loads_per_thread) {
    case 1: fn = (const void *)latency_kernel<1>; break;
    case 2: fn = (const void *)latency_kernel<2>; break;
    case 4: fn = (const void *)latency_kernel<4>; break;
    case 8: fn = (const void *)latency_kernel<8>; break;
    case 16: fn = (const void *)latency_kernel<16>; break;
    case 32: fn = (const void *)latency_kernel<32>; break;
    default: return -1;
    }
    return (int)hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(256), params, 0,
                                static_cast<hipStream_t>(stream));
}

}  // extern "C"
