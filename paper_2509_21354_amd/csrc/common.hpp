// Shared device helpers of the kvev kernels (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvev.h"

namespace kvev {

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 bits (lo in bits 0..15), round to nearest even, in
// one v_cvt_pk_bf16_f32 (gfx950 converts in hardware; NaN stays NaN).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_hw_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw_t));
}

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }

template <typename T> struct Storage;
template <> struct Storage<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Storage<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// N consecutive elements of storage type T -> fp32 registers, with the widest
// loads the alignment allows (the caller guarantees N*sizeof(T)-byte alignment
// up to 16 bytes).
template <typename T, int N> struct VecLoad;
template <> struct VecLoad<float, 4> {
    static __device__ __forceinline__ void run(const float *p, float (&o)[4])
    {
        float4 v = *reinterpret_cast<const float4 *>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
};
template <> struct VecLoad<float, 8> {
    static __device__ __forceinline__ void run(const float *p, float (&o)[8])
    {
        float4 a = reinterpret_cast<const float4 *>(p)[0];
        float4 b = reinterpret_cast<const float4 *>(p)[1];
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
        o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};
template <> struct VecLoad<bf16_t, 4> {
    static __device__ __forceinline__ void run(const bf16_t *p, float (&o)[4])
    {
        uint2 v = *reinterpret_cast<const uint2 *>(p);
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
    }
};
template <> struct VecLoad<bf16_t, 8> {
    static __device__ __forceinline__ void run(const bf16_t *p, float (&o)[8])
    {
        uint4 v = *reinterpret_cast<const uint4 *>(p);
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
};

// N consecutive elements kept in their raw register form (a 16-byte load is 4
// registers, not 8) until they are used.
// load_stream: the same load with the non-temporal hint, for cache rows that are read once per launch.  A plain
// streaming kernel reads 7.3 TB/s with the hint against 6.4 TB/s without on this chip.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <typename T, int N> struct Raw;
template <> struct Raw<bf16_t, 8> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void load_stream(const bf16_t *p)
    {
        const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        v = make_uint4(r[0], r[1], r[2], r[3]);
    }
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
};
template <> struct Raw<bf16_t, 4> {
    uint2 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint2 *>(p); }
    __device__ __forceinline__ void load_stream(const bf16_t *p)
    {
        const u32x2_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p));
        v = make_uint2(r[0], r[1]);
    }
    __device__ __forceinline__ void get(float (&o)[4]) const
    {
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
    }
};
template <> struct Raw<float, 4> {
    float4 v;
    __device__ __forceinline__ void load(const float *p) { v = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void load_stream(const float *p)
    {
        const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        v = make_float4(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[2]), __uint_as_float(r[3]));
    }
    __device__ __forceinline__ void get(float (&o)[4]) const { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
};
template <> struct Raw<float, 8> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p)
    {
        a = reinterpret_cast<const float4 *>(p)[0];
        b = reinterpret_cast<const float4 *>(p)[1];
    }
    __device__ __forceinline__ void load_stream(const float *p)
    {
        const u32x4_t r0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        const u32x4_t r1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p) + 1);
        a = make_float4(__uint_as_float(r0[0]), __uint_as_float(r0[1]), __uint_as_float(r0[2]), __uint_as_float(r0[3]));
        b = make_float4(__uint_as_float(r1[0]), __uint_as_float(r1[1]), __uint_as_float(r1[2]), __uint_as_float(r1[3]));
    }
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};

// 16-byte load through a buffer descriptor: address = descriptor base (SGPRs) +
// voff (one VGPR, shared by every load of the lane) + soff (SGPR or constant),
// with the constant part of voff folded into the instruction's immediate.  Keeps
// per-load 64-bit addresses out of the vector registers; a load past the
// descriptor's size returns zeros instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00027000);
}
template <typename V> __device__ __forceinline__ V buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff)
{
    const u32x4_t raw = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, (int)soff, 0);
    return __builtin_bit_cast(V, raw);
}
// The same with the non-temporal hint: for data read once, so that it does not push re-used lines out of L2.
template <typename V> __device__ __forceinline__ V buffer_load16_nt(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, uint32_t soff)
{
    const u32x4_t raw = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, (int)soff, 2);
    return __builtin_bit_cast(V, raw);
}

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// sum over the 16 lanes of a lane group (lanes that share lane/16)
__device__ __forceinline__ float group16_sum(float v)
{
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8);
    return v;
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }

// exact (erf) GELU in fp32
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

}  // namespace kvev
