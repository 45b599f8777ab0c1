// Wave64 / workgroup primitives used by the libtagc kernels (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tagc {

__device__ inline uint32_t lane_id() { return __lane_id(); }

template <typename T>
__device__ inline T wave_incl_scan(T v)
{
    const uint32_t l = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if (l >= uint32_t(d)) v += o;
    }
    return v;
}

// 32-bit inclusive scan on the VALU alone (DPP row shifts, then the two row broadcasts).
// A row shift reads zero where it has no source lane; a broadcast leaves the rows it is
// masked off from unchanged (they add the zero passed as the old value).
template <int CTRL>
__device__ inline uint32_t dpp_shr_add(uint32_t x)
{
    return x + uint32_t(__builtin_amdgcn_update_dpp(0, int(x), CTRL, 0xF, 0xF, true));
}
template <int CTRL, int ROW_MASK>
__device__ inline uint32_t dpp_bcast_add(uint32_t x)
{
    return x + uint32_t(__builtin_amdgcn_update_dpp(0, int(x), CTRL, ROW_MASK, 0xF, false));
}
template <>
__device__ inline uint32_t wave_incl_scan<uint32_t>(uint32_t x)
{
    x = dpp_shr_add<0x111>(x);          // row_shr:1
    x = dpp_shr_add<0x112>(x);          // row_shr:2
    x = dpp_shr_add<0x114>(x);          // row_shr:4
    x = dpp_shr_add<0x118>(x);          // row_shr:8
    x = dpp_bcast_add<0x142, 0xA>(x);   // row_bcast:15 into rows 1 and 3
    x = dpp_bcast_add<0x143, 0xC>(x);   // row_bcast:31 into rows 2 and 3
    return x;
}

template <typename T>
__device__ inline T wave_sum(T v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Exclusive scan over the NW*64 threads of a workgroup in thread order.  `smem` holds NW
// entries and may be reused after the call returns.
template <typename T, int NW>
__device__ inline T block_excl_scan(T v, T *total, T *smem)
{
    const uint32_t w = threadIdx.x >> 6, l = threadIdx.x & 63;
    T inc = wave_incl_scan(v);
    if (l == 63) smem[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        T x = smem[i];
        if (uint32_t(i) < w) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

template <typename T, int NW>
__device__ inline T block_sum(T v, T *smem)
{
    const uint32_t w = threadIdx.x >> 6, l = threadIdx.x & 63;
    T s = wave_sum(v);
    if (l == 0) smem[w] = s;
    __syncthreads();
    T tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) tot += smem[i];
    __syncthreads();
    return tot;
}

// float add on an LDS word.  The native LDS float atomic runs at about one lane per three
// clocks on this hardware (measured: 192 clocks per wave instruction against 6 for the
// integer ones), so the add is done with an integer compare-and-swap instead; collisions
// are rare in every use here, so the loop almost always runs once.
__device__ inline void lds_add_f32(float *p, float v)
{
    uint32_t *w = reinterpret_cast<uint32_t *>(p);
    uint32_t old = *w, assumed;
    do {
        assumed = old;
        old = atomicCAS(w, assumed, __float_as_uint(__uint_as_float(assumed) + v));
    } while (old != assumed);
}

// Streaming accesses: data that is read or written once and not touched again by the same
// kernel.  The non-temporal hint keeps such lines from displacing what the caches are for
// (measured on a 17-stream sum: 5.3 -> 5.9 TB/s, the rate of a pure read).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ inline uint4 ld_stream(const uint4 *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ inline float4 ld_stream(const float4 *p)
{
    const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ inline void st_stream(uint4 *p, uint4 v)
{
    const u32x4_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<u32x4_t *>(p));
}

__device__ inline void st_stream(float4 *p, float4 v)
{
    const f32x4_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<f32x4_t *>(p));
}

// bit p of the result = nibble p of x is not 0 (4-bit Index counters -> Index bits)
__device__ inline uint32_t nibbles_set(uint32_t x)
{
    x |= x >> 2;
    x |= x >> 1;
    x &= 0x11111111u;  // bit 4p = nibble p != 0
    x = (x | (x >> 3)) & 0x03030303u;
    x = (x | (x >> 6)) & 0x000F000Fu;
    return (x | (x >> 12)) & 0xFFu;
}

// float32 -> bfloat16 bits, round to nearest, ties to even; a NaN keeps a mantissa bit
__device__ inline uint32_t round_to_bf16(float x)
{
    const uint32_t b = __float_as_uint(x);
    if ((b & 0x7F800000u) == 0x7F800000u && (b & 0x007FFFFFu)) return (b >> 16) | 0x0040u;
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// Waits until every vector memory operation this thread has issued -- stores and atomics
// without a return value included -- has been acknowledged by the memory system.  Used
// before a workgroup announces, through another device-scope atomic, that its updates are
// there: a workgroup-scope release fence does not wait for them (it compiles to no wait
// on the vector memory counter), so the announcement could overtake the updates; and a
// device-scope release fence would also write back every dirty line of the L2, at many
// times the cost.  (s_waitcnt vmcnt(0); the other counters are left alone.)
__device__ inline void wait_own_memory_ops()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

__device__ inline uint64_t ld_agent(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace tagc
