// libpa device helpers: constants, element-type traits, cross-lane sums, streaming loads and stores.
#ifndef PA_PA_COMMON_HPP
#define PA_PA_COMMON_HPP

#include <hip/hip_runtime.h>

#include <stdint.h>

#include <type_traits>

#include "pa.h"

namespace {


constexpr int kWave = 64;
// Chunks whose loads are written together per trip of the streaming loop.  The compiler
// schedules the loads just in time whatever the source says (a few in flight per wave, the
// rest of the latency is covered by the other resident waves), and measured on MI355X that is
// what the memory side likes: one chunk per trip is as fast as two at the OPT-13B shape
// (170 us) and 2% faster at configs 4 and 5; four per trip is slower everywhere.  In the
// split-context kernel, where fewer waves work on one range, two per trip win (config 4 at
// 512-token partitions: 194 against 201 us).
constexpr int kChunksPerTrip = 1;
constexpr int kPartChunksPerTrip = 2;
constexpr float kLog2e = 1.4426950408889634f;
// running-maximum start value: finite, so that (m - m) is 0 and never NaN
constexpr float kNegBig = -3.0e38f;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// ---- cross-lane sums ------------------------------------------------------
// DPP controls: quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  Applied in this order they
// form a butterfly over 4, 8 and 16 consecutive lanes; every lane ends with
// the same bits because each step adds the same two partial sums.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, (int)as_u32(x), CTRL, 0xf, 0xf, true);
    return x + as_f32((uint32_t)y);
}

template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
    static_assert(LANES == 8 || LANES == 16 || LANES == 32, "lanes per token row");
    x = dpp_add<0xB1>(x);
    x = dpp_add<0x4E>(x);
    x = dpp_add<0x141>(x);
    if (LANES >= 16) x = dpp_add<0x140>(x);
    if (LANES >= 32) x += __shfl_xor(x, 16);
    return x;
}

// ---- element types -------------------------------------------------------
// A lane always holds one 16-byte fragment of a token row: 8 two-byte
// elements or 4 floats.
template <int DT> struct Traits;

template <> struct Traits<PA_F32> {
    static constexpr int E = 4, EPL = 4;
    static constexpr bool FENCE_AXPY = false;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        acc = __builtin_fmaf(as_f32(k.x), as_f32(q.x), acc);
        acc = __builtin_fmaf(as_f32(k.y), as_f32(q.y), acc);
        acc = __builtin_fmaf(as_f32(k.z), as_f32(q.z), acc);
        acc = __builtin_fmaf(as_f32(k.w), as_f32(q.w), acc);
        return acc;
    }
    static __device__ __forceinline__ void axpy(float (&acc)[4], float p, const uint4 &v)
    {
        acc[0] = __builtin_fmaf(p, as_f32(v.x), acc[0]);
        acc[1] = __builtin_fmaf(p, as_f32(v.y), acc[1]);
        acc[2] = __builtin_fmaf(p, as_f32(v.z), acc[2]);
        acc[3] = __builtin_fmaf(p, as_f32(v.w), acc[3]);
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[4])
    {
        return make_uint4(as_u32(x[0]), as_u32(x[1]), as_u32(x[2]), as_u32(x[3]));
    }
};

template <> struct Traits<PA_F16> {
    static constexpr int E = 2, EPL = 8;
    static constexpr bool FENCE_AXPY = false;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        // products of two halves are exact in fp32; accumulation is fp32
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.x), __builtin_bit_cast(half2_t, q.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.y), __builtin_bit_cast(half2_t, q.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.z), __builtin_bit_cast(half2_t, q.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, k.w), __builtin_bit_cast(half2_t, q.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void axpy2(float &a0, float &a1, float p, uint32_t v)
    {
        half2_t h = __builtin_bit_cast(half2_t, v);
        a0 = __builtin_fmaf(p, (float)h.x, a0);
        a1 = __builtin_fmaf(p, (float)h.y, a1);
    }
    static __device__ __forceinline__ void axpy(float (&acc)[8], float p, const uint4 &v)
    {
        axpy2(acc[0], acc[1], p, v.x);
        axpy2(acc[2], acc[3], p, v.y);
        axpy2(acc[4], acc[5], p, v.z);
        axpy2(acc[6], acc[7], p, v.w);
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        half2_t h;
        h.x = (_Float16)a;   // round to nearest even
        h.y = (_Float16)b;
        return __builtin_bit_cast(uint32_t, h);
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[8])
    {
        return make_uint4(pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7]));
    }
};

template <> struct Traits<PA_BF16> {
    static constexpr int E = 2, EPL = 8;
    static constexpr bool FENCE_AXPY = true;
    static __device__ __forceinline__ float dot(const uint4 &k, const uint4 &q, float acc)
    {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void axpy2(float &a0, float &a1, float p, uint32_t v)
    {
        // a bfloat16 is the upper half of a float
        a0 = __builtin_fmaf(p, as_f32(v << 16), a0);
        a1 = __builtin_fmaf(p, as_f32(v & 0xffff0000u), a1);
    }
    static __device__ __forceinline__ void axpy(float (&acc)[8], float p, const uint4 &v)
    {
        axpy2(acc[0], acc[1], p, v.x);
        axpy2(acc[2], acc[3], p, v.y);
        axpy2(acc[4], acc[5], p, v.z);
        axpy2(acc[6], acc[7], p, v.w);
    }
    static __device__ __forceinline__ uint32_t rne(float f)
    {
        uint32_t u = as_u32(f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ uint4 pack(const float (&x)[8])
    {
        return make_uint4(rne(x[0]) | (rne(x[1]) << 16), rne(x[2]) | (rne(x[3]) << 16),
                          rne(x[4]) | (rne(x[5]) << 16), rne(x[6]) | (rne(x[7]) << 16));
    }
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// 16-byte load with the non-temporal hint: K/V bytes are used exactly once per
// call, and streaming them past the caches measurably raises the HBM rate.
__device__ __forceinline__ uint4 load16_stream(const char *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Streaming copies: data that passes through once is loaded and stored with
// the non-temporal hint (measured 6.4 TB/s of read+write traffic for block
// copies against 5.7 TB/s with plain accesses).
__device__ __forceinline__ u32x4_t load_frag_stream(const uint4 *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}
__device__ __forceinline__ void store_frag_stream(uint4 *p, u32x4_t v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(p));
}


} // namespace

#endif
