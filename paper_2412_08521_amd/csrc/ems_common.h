// Shared device-side helpers for the gfx950 EMS kernels: MFMA operand fragments, the
// accumulator's lane/register -> (row, column) map, and small wave utilities.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ems {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// One MFMA operand fragment is 16 bytes per lane whatever the element type.
//
// v_mfma_f32_32x32x16_bf16: lane l supplies row (A) / column (B) l % 32 and the 8
// consecutive k-elements starting at 8 * (l / 32).
// v_mfma_f32_32x32x2_f32:   lane l supplies row / column l % 32 and k-element l / 32; a
// 16-byte fragment (4 floats) feeds 4 such instructions, component t to instruction t.
// In both cases lane l reads the 16 bytes at byte offset  f * 32 + (l / 32) * 16  of its
// row for fragment f, and A and B fragments pair up the same head_dim elements, which is
// all a dot product needs.
typedef i32x4_t frag_t;

template <typename T> struct Elem;
template <> struct Elem<bf16_t> { static constexpr int kBytes = 2; };
template <> struct Elem<float> { static constexpr int kBytes = 4; };

template <typename T, int D> struct Tile {
    static constexpr int kRowBytes = D * Elem<T>::kBytes;
    static constexpr int kFrags = kRowBytes / 32;          // fragments per row per lane
    static constexpr int kLdsStride = kRowBytes + 16;      // padded row pitch in LDS (bytes)
    static constexpr int kChunksPerRow = kRowBytes / 16;   // 16-byte chunks per row
};

template <typename T>
__device__ __forceinline__ void mma(f32x16_t& acc, const frag_t& a, const frag_t& b);

template <>
__device__ __forceinline__ void mma<bf16_t>(f32x16_t& acc, const frag_t& a, const frag_t& b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                  __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mma<float>(f32x16_t& acc, const frag_t& a, const frag_t& b)
{
    const f32x4_t af = __builtin_bit_cast(f32x4_t, a);
    const f32x4_t bf = __builtin_bit_cast(f32x4_t, b);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[0], bf[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[1], bf[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[2], bf[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[3], bf[3], acc, 0, 0, 0);
}

// First product of a chain: the accumulator starts from zero.
template <typename T>
__device__ __forceinline__ void mma_first(f32x16_t& acc, const frag_t& a, const frag_t& b)
{
    acc = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    mma<T>(acc, a, b);
}

// 32x32 accumulator: register r of lane l holds output row acc_row(r, l / 32) (the A
// operand's row) and output column l % 32 (the B operand's column).
__device__ __forceinline__ constexpr int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ frag_t zero_frag() { return frag_t{0, 0, 0, 0}; }

// 16-byte global load, or zeros when `ok` is false (never touches memory then).
__device__ __forceinline__ frag_t load_frag_or_zero(const void* base, size_t byte_off, bool ok)
{
    if (!ok) return zero_frag();
    return *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(base) + byte_off);
}

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return (float)x; }

}  // namespace ems
