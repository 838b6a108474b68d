// Measurement kernels declared in include/ems_probe.h: the matrix pipe's and the memory
// system's own ceilings on the machine the benchmark runs on.
#include "../../include/ems.h"
#include "../../include/ems_probe.h"
#include "ems_common.h"

namespace ems {

__global__ __launch_bounds__(256) void probe_mfma_kernel(float* sink, int iters)
{
    const int lane = threadIdx.x % kWave;
    // operands that are neither zero nor denormal; their values do not matter
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (bf16_t)(1.0f + 0.001f * (float)(lane + i)); b[i] = (bf16_t)(0.5f - 0.002f * (float)(lane - i)); }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
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

int ems_probe_mfma(int32_t blocks, int32_t iters, float* sink, void* hip_stream)
{
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || !sink) return EMS_ERR_INVALID_ARG;
    hipLaunchKernelGGL(ems::probe_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), sink, iters);
    return hipGetLastError() == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream)
{
    if (!src || !dst || bytes == 0 || (bytes % 16) != 0 || ((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0)
        return EMS_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 256u * 32u ? want : 256u * 32u);   // 32 blocks per compute unit
    hipLaunchKernelGGL(ems::probe_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const ems::frag_t*>(src), static_cast<ems::frag_t*>(dst), n16);
    return hipGetLastError() == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

}  // extern "C"
