// Element load/store helpers: float or bfloat16 storage, float arithmetic.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace lpm {

struct bf16_t { uint16_t bits; };   // storage only

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

// Streaming accesses: data touched once per kernel (parameters in the update, the fp32 gradient of a large FC
// layer) is read and written with the non-temporal hint so it does not displace reusable lines from the caches.
typedef float lpm_f4 __attribute__((ext_vector_type(4)));
typedef unsigned int lpm_u2 __attribute__((ext_vector_type(2)));
typedef unsigned int lpm_u4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld_stream(const float4* a) {
    const lpm_f4 t = __builtin_nontemporal_load(reinterpret_cast<const lpm_f4*>(a));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint4 ld_stream(const uint4* a) {
    const lpm_u4 t = __builtin_nontemporal_load(reinterpret_cast<const lpm_u4*>(a));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st_stream(float4* a, float4 x) {
    const lpm_f4 t = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(t, reinterpret_cast<lpm_f4*>(a));
}
__device__ __forceinline__ void st_stream(uint2* a, uint2 x) {
    const lpm_u2 t = {x.x, x.y};
    __builtin_nontemporal_store(t, reinterpret_cast<lpm_u2*>(a));
}

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (each with its own L2), so give
// every XCD one contiguous range of tiles.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
    const int per = nblocks >> 3, rem = nblocks & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    return xcd * per + min(xcd, rem) + idx;
}

__device__ __forceinline__ float ld(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld(const bf16_t* p, int64_t i) { return bf2f(p[i].bits); }
__device__ __forceinline__ void st(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st(bf16_t* p, int64_t i, float v) { p[i].bits = f2bf(v); }

}  // namespace lpm
