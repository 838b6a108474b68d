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

// ---- DPP lane permutations (ALU latency, no LDS round trip)
template <int kCtrl>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, false));
}
template <int kCtrl>
__device__ __forceinline__ int dpp_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xf, 0xf, false);
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i inside each group of 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i inside each row of 16

template <bool kMax> __device__ __forceinline__ float comb(float a, float b) { return kMax ? fmaxf(a, b) : a + b; }
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}


// Sum over the kLpr consecutive lanes that hold one row (kLpr = 8, 16 or 32); every lane of
// the group gets the total.
template <int kLpr>
__device__ __forceinline__ float group_sum(float v)
{
    v += dpp_f<kDppXor1>(v);
    v += dpp_f<kDppXor2>(v);
    v += dpp_f<kDppHalfMirror>(v);
    if constexpr (kLpr >= 16) v += dpp_f<kDppMirror>(v);
    if constexpr (kLpr >= 32) v += __shfl_xor(v, 16);
    return v;
}

}  // namespace ems
