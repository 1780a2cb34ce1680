// Device helpers shared by the decode-attention kernels.
#pragma once

#include <math.h>

#include "kv_internal.h"

namespace kvdec {

constexpr float kNegInf = -INFINITY;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)f32_to_bf16_bits(f); }

// two fp32 -> packed bf16 pair (lo in bits 15:0), round to nearest even, one hardware convert
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

__device__ __forceinline__ bf16x8 as_bf16x8(kv_u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[8])
{
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x);
    f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z);
    f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

// 2^x by the hardware instruction (exact at -inf -> 0; results below the normal range flush).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Combine (m2, l2, a2[]) into (m, l, a[]); all maxima may be -inf (empty partials).
template <int N>
__device__ __forceinline__ void combine(float& m, float& l, float (&a)[N], float m2, float l2,
                                        const float (&a2)[N])
{
    const float mn = fmaxf(m, m2);
    const float ms = (mn == kNegInf) ? 0.f : mn;
    const float c1 = exp2f(m - ms), c2 = exp2f(m2 - ms);
    l = l * c1 + l2 * c2;
#pragma unroll
    for (int e = 0; e < N; ++e) a[e] = a[e] * c1 + a2[e] * c2;
    m = mn;
}

// Data that travels between workgroups which may run on different XCDs, each with its own L2, is
// written and read with relaxed device-scope atomic accesses of 64 bits, which the hardware serves
// at the device's point of coherence (write-through stores, loads that bypass the local caches).
// Ordering comes from waiting for the stores' acknowledgement (s_waitcnt vmcnt(0)) before an arrival
// counter is touched, not from cache-wide fences.
__device__ __forceinline__ void st_coherent2(float* p, float x, float y)
{
    const unsigned long long bits =
        (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), bits, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x2 ld_coherent2(const float* p)
{
    const unsigned long long bits = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return f32x2{__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32))};
}

}  // namespace kvdec
