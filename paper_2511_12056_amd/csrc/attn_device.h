// Device-side vector types and wavefront helpers shared by the attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

namespace pda {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T) T __attribute__((address_space(3)))*

// Lanes l and l^32 hold the two halves of one query's keys.  v_permlane32_swap hands every lane
// both halves' values (one in each result register), so max and sum need no select.
__device__ __forceinline__ float pair_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// max of three, as one instruction.  Written in assembly so that it stays where it is put and so
// that no NaN-quieting copies of the operands are added (callers pass finite scores or -inf).
__device__ __forceinline__ float max3_f32(float a, float b, float c) {
    float r;
    asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);     // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(unsigned, h);
}

// Streaming (non-temporal) 16- and 8-byte accesses for data that is touched once: they leave the
// caches to data that is reused and measurably raise the rate of the HBM-bound kernels.
__device__ __forceinline__ float4 nt_load4(const float4* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store4(float4* p, const float4& a) {
    const f32x4 v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}
__device__ __forceinline__ void nt_store2(uint2* p, unsigned lo, unsigned hi) {
    const u32x2 v = {lo, hi};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
}

// Compile-time loop: f(std::integral_constant<int, I>) for I in [I0, N).
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

}  // namespace pda
