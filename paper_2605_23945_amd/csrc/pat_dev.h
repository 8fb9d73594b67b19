// Device-side helpers shared by the HIP kernels of the decode step (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));     // a 16-byte fragment as a native vector

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even; finite inputs and infinities (NaN is mapped to a quiet NaN)
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// the two bf16 values held in one 32-bit word, widened
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// x = hi + lo + O(2^-17 |x|), both bf16: the operand split that keeps fp32-class
// accuracy on the bf16 matrix cores.
__device__ __forceinline__ void split_bf16(float v, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16(v);
    lo = f32_to_bf16(v - bf16_to_f32(hi));
}

// Packed operand layouts for v_mfma_f32_16x16x32_bf16.  A k-step is 32
// consecutive k; lane l of a wave holds 8 consecutive k (group g = l / 16) of
// row r = l % 16, i.e. one 16-byte vector; a (16-row tile, k-step) block is the
// 64 lanes' vectors back to back = 1 KiB.
//   vector index of (tile, kstep, lane) = (tile * KS + kstep) * 64 + lane
// Offset in bf16 elements of element (row, k) of a [rows, K] operand:
__device__ __host__ __forceinline__ int64_t packed_elem_offset(int row, int k, int KS)
{
    int tile = row >> 4, r = row & 15, ks = k >> 5, g = (k & 31) >> 3, j = k & 7;
    return ((((int64_t)tile * KS + ks) * 64 + g * 16 + r) << 3) + j;
}

// Agent-scope (write-through) stores and loads: data that another workgroup of the SAME launch reads after a
// device-wide barrier is written with these, so that no cache-wide write-back is needed; the reader uses
// plain loads provided the address was not read earlier in the launch (no stale line can exist then).
__device__ __forceinline__ void store4_agent(void *p, uint32_t v)
{
    __hip_atomic_store(reinterpret_cast<uint32_t *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store8_agent(void *p, uint64_t v)
{
    __hip_atomic_store(reinterpret_cast<uint64_t *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store16_agent(void *p, uint4 v)
{
    store8_agent(p, (uint64_t)v.x | ((uint64_t)v.y << 32));
    store8_agent(reinterpret_cast<char *>(p) + 8, (uint64_t)v.z | ((uint64_t)v.w << 32));
}
__device__ __forceinline__ void storef4_agent(float *p, float4 v)
{
    store8_agent(p, (uint64_t)__float_as_uint(v.x) | ((uint64_t)__float_as_uint(v.y) << 32));
    store8_agent(p + 2, (uint64_t)__float_as_uint(v.z) | ((uint64_t)__float_as_uint(v.w) << 32));
}
__device__ __forceinline__ void storef_agent(float *p, float v) { store4_agent(p, __float_as_uint(v)); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

}  // namespace pat
