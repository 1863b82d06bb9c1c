// Storage helpers shared by the bandwidth-bound kernels: fp32 / bf16 element and 16-byte vector access.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dr {
namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float((uint32_t)u << 16); }
// two fp32 -> two bf16 in one word, round to nearest even, NaN stays NaN (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }

// s^-beta for the normalisation layers (Eq. (3)): beta = 0.75 as rsqrt(s) * sqrt(rsqrt(s)), 1 ulp hardware approximations
__device__ __forceinline__ float pow_neg_beta(float s, float beta, bool b075)
{
    if (b075) {
        const float r = __builtin_amdgcn_rsqf(s);
        return r * __builtin_amdgcn_sqrtf(r);
    }
    return powf(s, -beta);
}

template <typename T> struct Store;
template <> struct Store<float> {
    static constexpr int VN = 4;   // elements per 16 bytes
    static __device__ __forceinline__ float ld(const float* p) { return *p; }
    static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void ldv(const float* p, float* v)
    {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ void stv(float* p, const float* v)
    {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct Store<uint16_t> {
    static constexpr int VN = 8;
    static __device__ __forceinline__ float ld(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void ldv(const uint16_t* p, float* v)
    {
        const uint4 t = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ void stv(uint16_t* p, const float* v)
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline unsigned blocks_for(size_t items, int per_block, size_t cap = 1u << 20)
{
    size_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    return (unsigned)(b > cap ? cap : b);
}

}  // namespace
}  // namespace dr
