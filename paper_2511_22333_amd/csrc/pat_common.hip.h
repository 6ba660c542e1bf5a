// Device-side helpers shared by the forward and merge kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pat_internal.h"

namespace pat {

constexpr int kHeadDim = 128;
constexpr int kPage = 16;
constexpr int kWave = 64;

struct F16 {};    // tag types: element type of q / K / V / out
struct BF16 {};

template <typename T> struct Elem;
template <> struct Elem<F16> {
    using raw = _Float16;
    static __device__ __forceinline__ float to_f32(uint16_t bits)
    {
        return (float)__builtin_bit_cast(_Float16, bits);
    }
    static __device__ __forceinline__ uint16_t from_f32(float x)
    {
        return __builtin_bit_cast(uint16_t, (_Float16)x);      // round to nearest even
    }
};
template <> struct Elem<BF16> {
    static __device__ __forceinline__ float to_f32(uint16_t bits)
    {
        return __builtin_bit_cast(float, (uint32_t)bits << 16);
    }
    static __device__ __forceinline__ uint16_t from_f32(float x)
    {
        uint32_t u = __builtin_bit_cast(uint32_t, x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN
        u += 0x7fffu + ((u >> 16) & 1u);                                            // RNE
        return (uint16_t)(u >> 16);
    }
};

// The schedule is read-only while a kernel runs: unit records are read through the constant
// address space, which makes their (workgroup-uniform) loads scalar loads whatever else the
// kernel stores in between.
typedef __attribute__((address_space(4))) DevUnit ConstDevUnit;

// The whole 128-byte unit record in scalar registers: two scalar loads and one wait, issued as
// the first thing a workgroup does.  Every field a tile needs to send out its first K/V and q
// loads is then there after ONE round trip; left to the compiler, the record's second cache line
// (the inlined page and request ids) is fetched only when a tile first touches it, behind the
// branches on the tile id, which costs a second dependent round trip before any data is asked for.
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
struct UnitRec {
    i32x4 e0, e1, h, p0, p1, rq;            // six 16-byte pieces of the record's first 96 bytes
    __device__ __forceinline__ int req_off() const { return e0[0]; }
    __device__ __forceinline__ int n_req() const { return e0[1]; }
    __device__ __forceinline__ int page_off() const { return e0[2]; }
    __device__ __forceinline__ int n_pages() const { return e0[3]; }
    __device__ __forceinline__ int kv_len() const { return e1[0]; }
    __device__ __forceinline__ int row_begin() const { return e1[1]; }
    __device__ __forceinline__ int n_rows() const { return e1[2]; }
    __device__ __forceinline__ int tile() const { return e1[3]; }
    __device__ __forceinline__ int kvh0() const { return h[0]; }
    __device__ __forceinline__ int n_heads() const { return h[1]; }
    // inlined ids: pages 0..7 and requests 0..3 of the entry
    __device__ __forceinline__ int page(int i) const { return i < 4 ? p0[i] : p1[i - 4]; }
    __device__ __forceinline__ int req(int i) const { return rq[i]; }
};
static_assert(offsetof(DevUnit, kvh0) == 32 && offsetof(DevUnit, page0) == 48 &&
              offsetof(DevUnit, page4) == 64 && offsetof(DevUnit, req0) == 80, "UnitRec pieces");
__device__ __forceinline__ void unit_fetch(const DevUnit *p, UnitRec &r)
{
    asm volatile("s_load_dwordx4 %0, %6, 0x0\n\ts_load_dwordx4 %1, %6, 0x10\n\t"
                 "s_load_dwordx4 %2, %6, 0x20\n\ts_load_dwordx4 %3, %6, 0x30\n\t"
                 "s_load_dwordx4 %4, %6, 0x40\n\ts_load_dwordx4 %5, %6, 0x50\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(r.e0), "=&s"(r.e1), "=&s"(r.h), "=&s"(r.p0), "=&s"(r.p1), "=&s"(r.rq)
                 : "s"(p)
                 : "memory");
}

// Arguments common to every forward kernel.
struct FwdArgs {
    const DevUnit *units;         // one per workgroup, launch order
    const int32_t *req_ids;
    const int32_t *req_slot;
    const int32_t *page_ids;
    const uint16_t *q;            // [B][Hq][d]
    const uint16_t *k_pool;
    const uint16_t *v_pool;
    int64_t stride_page, stride_token, stride_head;   // elements
    uint16_t *out;                // [B][Hq][d]
    float *lse;                   // [B][Hq] or nullptr
    float *part_o;                // [slots][Hq][d]
    float *part_lse;              // [slots][Hq]
    float scale;                  // softmax scale
    int32_t Hq, Hkv, G;
    unsigned long long *trace;    // optional [units][8] timeline records, or nullptr
    int32_t n_units;              // unit records
    int32_t queue_begin;          // units from here on are taken from a queue by persistent workgroups
    int32_t queue_workers;        // how many of those (the last workgroups of the grid); 0: no queue
    int32_t *queue_ctr;           // [0]: next queued unit, [1]: workers that have left; both 0 between launches
    // merge fused into the launch (fuse_mode != 0)
    int32_t fuse_mode, n_merge, spin_limit;
    const int32_t *req_midx;      // parallel to req_ids: merge record of the request or -1
    const int32_t *merge_rec;     // 128-byte merge records
    const int32_t *req_slot_ids;
    int32_t *merge_state;         // [n_merge][Hkv] task state words
    int32_t unit_base;            // unit of workgroup 0 (the 16-row kernel of a two-kernel launch)
    const DevWorker *workers;     // launches with wavefront items: one record per persistent workgroup
    const DevWaveItem *wave_items;
};

// Timeline marks 0..3 of a workgroup (time on the 100 MHz constant clock).  The times are kept
// in scalar registers and written when the tile function ends: a store in the middle of a
// tile would make the compiler wait for it (and with it for every load in flight) before it
// reuses the store's registers, which changes the very timing the marks are there to show.
struct TraceMarks {
    unsigned long long t[4] = {0, 0, 0, 0};
    __device__ __forceinline__ void mark(const FwdArgs &a, int k)
    {
        if (a.trace) t[k] = wall_clock64();
    }
    // thread 0 of each 256-thread half writes the marks it took
    __device__ __forceinline__ void flush(const FwdArgs &a, int unit) const
    {
        if (a.trace && (threadIdx.x & 255) == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (t[k]) a.trace[8ull * unit + 4 + k] = t[k];
        }
    }
};

struct MergeArgs {
    const int32_t *merge_rec;     // one record per request with more than one partial
    const int32_t *req_slot_ids;  // full slot lists (for what a record does not hold)
    const float *part_o;
    const float *part_lse;
    uint16_t *out;
    float *lse;
    int32_t n_merge, Hq;
    int32_t long_lists;           // mean partials per listed request >= 8: one wavefront per head
};

// ---- matrix-core helpers -------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Operands are 8 consecutive 16-bit elements of the contraction dimension per lane.
//   16x16x32: A[i][k], B[k][j]: lane = (i or j) + 16 * (k / 8); D[i][j]: lane = j + 16 * (i / 4),
//             register i % 4.
//   32x32x16: lane = (i or j) + 32 * (k / 8); D[i][j]: lane = j + 32 * ((i / 4) % 2),
//             register (i % 4) + 4 * (i / 8).
template <typename T> struct Mma;
template <> struct Mma<BF16> {
    static __device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};
template <> struct Mma<F16> {
    static __device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        f16x2 v = {(_Float16)lo, (_Float16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};

__device__ __forceinline__ u32x4 load16(const uint16_t *p)
{
    return *reinterpret_cast<const u32x4 *>(p);
}
// K and V are read once per launch: a non-temporal load keeps them from displacing what the
// caches are useful for, and streams measurably faster from HBM on this GPU.
__device__ __forceinline__ u32x4 load16_stream(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// Partial rows are written once and read by another kernel: stored non-temporally they leave
// the L2 at once instead of waiting for the write-back at the kernel's end.
__device__ __forceinline__ void store16_stream(float *p, float x, float y, float z, float w)
{
    __builtin_nontemporal_store(f32x4{x, y, z, w}, reinterpret_cast<f32x4 *>(p));
}

// Partials that are merged INSIDE the launch that writes them (by a workgroup on another XCD, whose
// L2 is not coherent with this one's): stored and loaded at agent scope, i.e. written through and
// read past the L2s, so that an arrival counter can order them without flushing a whole L2 per
// workgroup (a device-wide fence does that, and costs more than the merge kernel it would save).
__device__ __forceinline__ void store16_agent(float *p, float x, float y, float z, float w)
{
    const f32x4 v = {x, y, z, w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store1_agent(float *p, float x)
{
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool AGENT>
__device__ __forceinline__ float load1(const float *p)
{
    return AGENT ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
}
template <bool AGENT>
__device__ __forceinline__ float4 load4(const float *p)
{
    if (!AGENT) return *reinterpret_cast<const float4 *>(p);
    return make_float4(load1<true>(p), load1<true>(p + 1), load1<true>(p + 2), load1<true>(p + 3));
}

// LDS the single forward kernel reserves.  The 16-row tiles run on 256-thread halves of the
// workgroup with half of it each; the packed tiles use all of it.
constexpr int kHalfSmemBytes = 36864;
constexpr int kFwdSmemBytes = 2 * kHalfSmemBytes + 5120;

// Write one finished row: 8 consecutive head-dim elements o[0..7] starting at c0, either as an
// fp32 partial (slot >= 0) or as the final output in the element type.
template <typename T>
__device__ __forceinline__ void store_row_chunk(const FwdArgs &a, int slot, int req, int head,
                                                int c0, const float *o, float lse, bool lse_lane)
{
    if (slot >= 0) {
        float *dst = a.part_o + ((int64_t)slot * a.Hq + head) * kHeadDim + c0;
        if (a.fuse_mode) {                              // uniform: merged inside this launch
            store16_agent(dst, o[0], o[1], o[2], o[3]);
            store16_agent(dst + 4, o[4], o[5], o[6], o[7]);
            if (lse_lane) store1_agent(a.part_lse + (int64_t)slot * a.Hq + head, lse);
        } else {
            store16_stream(dst, o[0], o[1], o[2], o[3]);
            store16_stream(dst + 4, o[4], o[5], o[6], o[7]);
            if (lse_lane) a.part_lse[(int64_t)slot * a.Hq + head] = lse;
        }
    } else {
        uint16_t *dst = a.out + ((int64_t)req * a.Hq + head) * kHeadDim + c0;
        uint32_t pk[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            pk[c] = (uint32_t)Elem<T>::from_f32(o[2 * c]) |
                    ((uint32_t)Elem<T>::from_f32(o[2 * c + 1]) << 16);
        *reinterpret_cast<uint4 *>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        if (a.lse && lse_lane) a.lse[(int64_t)req * a.Hq + head] = lse;
    }
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

}  // namespace pat
