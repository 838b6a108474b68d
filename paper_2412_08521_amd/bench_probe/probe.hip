// Measurement kernels declared in ems_probe.h: the matrix pipe's and the memory system's own
// ceilings on the machine the benchmark runs on.  Built into libems_probe.so, apart from the
// product library.
#include "ems_probe.h"
#include "../csrc/ems_common.h"

namespace ems {

__global__ __launch_bounds__(256) void probe_mfma_kernel(const frag_t* operands, float* sink, int iters)
{
    const int lane = threadIdx.x % kWave;
    // 8 A and 8 B fragments per lane: from the caller's buffer, or constants that are neither zero
    // nor denormal (their values do not matter)
    frag_t a[8], b[8];
    constexpr int kFragsInBuffer = 65536 / 16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (operands) {
            a[i] = operands[(threadIdx.x * 16 + i) % kFragsInBuffer];
            b[i] = operands[(threadIdx.x * 16 + 8 + i + blockIdx.x) % kFragsInBuffer];
        } else {
            bf16x8_t x, y;
#pragma unroll
            for (int e = 0; e < 8; ++e) { x[e] = (bf16_t)(1.0f + 0.001f * (float)(lane + e)); y[e] = (bf16_t)(0.5f - 0.002f * (float)(lane - e)); }
            a[i] = __builtin_bit_cast(frag_t, x); b[i] = __builtin_bit_cast(frag_t, y);
        }
    }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mma<bf16_t>(c0, a[i], b[i]);
            mma<bf16_t>(c1, a[i], b[(i + 1) & 7]);
            mma<bf16_t>(c2, a[i], b[(i + 2) & 7]);
            mma<bf16_t>(c3, a[i], b[(i + 3) & 7]);
        }
        if ((it & 63) == 63) { c0 = c0 * 0.f; c1 = c1 * 0.f; c2 = c2 * 0.f; c3 = c3 * 0.f; }   // stays finite
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const frag_t* src, frag_t* dst, size_t n16)
{
    // four 16-byte loads in flight per thread, each a fully coalesced wave-wide access
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const frag_t a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace ems

extern "C" {

int ems_probe_mfma(int32_t blocks, int32_t iters, const void* operands, float* sink, void* hip_stream)
{
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || !sink || ((uintptr_t)operands % 16) != 0) return -1;
    hipLaunchKernelGGL(ems::probe_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const ems::frag_t*>(operands), sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

int ems_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream)
{
    if (!src || !dst || bytes == 0 || (bytes % 16) != 0 || ((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0)
        return -1;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256u * 32u ? want : 256u * 32u);   // 32 blocks per compute unit
    hipLaunchKernelGGL(ems::probe_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const ems::frag_t*>(src), static_cast<ems::frag_t*>(dst), n16);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
