// Row-wise helpers shared by the merge, expansion and decode kernels: a cache row of D
// elements is handled as 16-byte pieces, one per lane.
#pragma once

#include "ems_common.h"

namespace ems {

// sum of squares of the 16-byte fragment's elements, in f32
template <typename T> __device__ __forceinline__ float frag_sumsq(const frag_t& f);
template <> __device__ __forceinline__ float frag_sumsq<bf16_t>(const frag_t& f)
{
    const bf16x8_t v = __builtin_bit_cast(bf16x8_t, f);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { const float x = (float)v[i]; s = __builtin_fmaf(x, x, s); }
    return s;
}
template <> __device__ __forceinline__ float frag_sumsq<float>(const frag_t& f)
{
    const f32x4_t v = __builtin_bit_cast(f32x4_t, f);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s = __builtin_fmaf(v[i], v[i], s);
    return s;
}

__device__ __forceinline__ float inv_norm(float sumsq) { return sumsq > 0.f ? 1.0f / sqrtf(sumsq) : 0.f; }

template <typename T> struct Pack;
template <> struct Pack<bf16_t> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void unpack(const frag_t& f, float (&x)[8])
    {
        const bf16x8_t v = __builtin_bit_cast(bf16x8_t, f);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = (float)v[i];
    }
    static __device__ __forceinline__ frag_t pack(const float (&x)[8])
    {
        bf16x8_t v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (bf16_t)x[i];      // round to nearest even
        return __builtin_bit_cast(frag_t, v);
    }
};
template <> struct Pack<float> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void unpack(const frag_t& f, float (&x)[4])
    {
        const f32x4_t v = __builtin_bit_cast(f32x4_t, f);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = v[i];
    }
    static __device__ __forceinline__ frag_t pack(const float (&x)[4])
    {
        f32x4_t v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = x[i];
        return __builtin_bit_cast(frag_t, v);
    }
};

}  // namespace ems
