// Per-head statistics of Sec. 4.1: sparsity rate (Eq. 3) and redundancy rate (Eq. 4).
//
// sparsity_kernel    one block per (batch, kv-head): Eq. 2 score of every position, then
//                    the smallest number of top scores whose mass reaches zeta of the total,
//                    found without sorting by an 8-bit-digit radix descent over the
//                    order-preserving integer image of the scores.  Masses are added as
//                    64-bit fixed-point integers, so the result does not depend on the
//                    order in which the atomics land.
// redundancy_kernel  for every token the best key-cosine x value-cosine against all EARLIER
//                    tokens: both cosines as MFMA contractions of raw rows scaled by
//                    reciprocal norms, running maximum per lane (the layout of the merge
//                    destination kernel with "centres" = the causal prefix).
// redundancy_count_kernel  tokens whose best redundancy reaches tau, per head.
#include "ems_common.h"
#include "ems_kernels.h"
#include "ems_rows.h"

namespace ems {

constexpr int kStatBlock = 1024;
constexpr int kStatWaves = kStatBlock / kWave;
constexpr double kMassOne = 1099511627776.0;   // 2^40: fixed-point image of the whole score mass

// scores are >= 0: their bit patterns already order like the values
__device__ __forceinline__ uint32_t score_key(float s) { return __float_as_uint(fmaxf(s, 0.f)); }

__global__ __launch_bounds__(kStatBlock) void sparsity_kernel(StatsArgs a)
{
    __shared__ float red[kStatWaves][2];
    __shared__ int cnt[256];
    __shared__ unsigned long long mass[256];
    __shared__ unsigned long long sh_total;
    __shared__ uint32_t sh_prefix;
    __shared__ unsigned long long sh_mass_above;
    __shared__ int sh_count_above;

    const int N = a.seq_len;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const float* glo = a.s_glo + (size_t)blockIdx.x * N;
    const float* loc = a.s_loc + (size_t)blockIdx.x * N;

    // Eq. 2 alignment factor, fixed-order sums
    float sg = 0.f, sl = 0.f;
    for (int j = tid; j < N; j += kStatBlock) { sg += glo[j]; sl += loc[j]; }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { sg += __shfl_xor(sg, o); sl += __shfl_xor(sl, o); }
    if (lane == 0) { red[wave][0] = sg; red[wave][1] = sl; }
    if (tid == 0) sh_total = 0ull;
    __syncthreads();
    float tot_g = 0.f, tot_l = 0.f;
    for (int w = 0; w < kStatWaves; ++w) { tot_g += red[w][0]; tot_l += red[w][1]; }
    const float align = tot_g > 0.f ? (tot_l / (float)N) / (tot_g / (float)N) : 0.f;

    // total of the Eq. 2 scores (float tree), then every score as a share of it in fixed point
    float st = 0.f;
    for (int j = tid; j < N; j += kStatBlock) st += fmaxf(glo[j] * align, loc[j]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) st += __shfl_xor(st, o);
    __syncthreads();
    if (lane == 0) red[wave][0] = st;
    __syncthreads();
    float tot_s = 0.f;
    for (int w = 0; w < kStatWaves; ++w) tot_s += red[w][0];
    const double to_fixed = tot_s > 0.f ? kMassOne / (double)tot_s : 0.0;

    unsigned long long part = 0ull;
    for (int j = tid; j < N; j += kStatBlock)
        part += (unsigned long long)((double)fmaxf(glo[j] * align, loc[j]) * to_fixed);
    atomicAdd(&sh_total, part);
    if (tid == 0) { sh_prefix = 0u; sh_mass_above = 0ull; sh_count_above = 0; }
    __syncthreads();
    // smallest integer mass that counts as "zeta of the total"
    const unsigned long long need_total = (unsigned long long)ceil((double)a.zeta * (double)sh_total);

    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int d = tid; d < 256; d += kStatBlock) { cnt[d] = 0; mass[d] = 0ull; }
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        for (int j = tid; j < N; j += kStatBlock) {
            const float s = fmaxf(glo[j] * align, loc[j]);
            const uint32_t key = score_key(s);
            if (shift < 24 && (key >> (shift + 8)) != prefix) continue;
            const int digit = (key >> shift) & 255;
            atomicAdd(&cnt[digit], 1);
            atomicAdd(&mass[digit], (unsigned long long)((double)s * to_fixed));
        }
        __syncthreads();
        if (tid == 0) {
            // walk the digits from the largest: stop in the one where the mass crosses
            unsigned long long m = sh_mass_above;
            int c = sh_count_above, d = 255;
            for (; d > 0; --d) {
                if (m + mass[d] >= need_total) break;
                m += mass[d];
                c += cnt[d];
            }
            sh_mass_above = m;
            sh_count_above = c;
            sh_prefix = (prefix << 8) | (uint32_t)d;
        }
        __syncthreads();
    }
    if (tid == 0) {
        // every score with the final key has the same value, hence the same fixed-point mass
        const uint32_t key = sh_prefix;
        const float s_star = __uint_as_float(key);
        const unsigned long long q = (unsigned long long)((double)s_star * to_fixed);
        const int equal = cnt[key & 255];
        const unsigned long long need = need_total > sh_mass_above ? need_total - sh_mass_above : 0ull;
        long long extra = q > 0ull ? (long long)((need + q - 1ull) / q) : (long long)equal;
        if (extra < 1) extra = 1;
        if (extra > equal) extra = equal;
        long long nk = (long long)sh_count_above + extra;
        if (sh_total == 0ull) nk = 1;                        // all scores zero: the first one already "reaches" zeta of 0
        if (nk > N) nk = N;
        if (nk < 1) nk = 1;
        a.p_out[blockIdx.x] = 1.0f - (float)((double)nk / (double)N);
        if (a.n_k_opt) a.n_k_opt[blockIdx.x] = (int32_t)nk;
    }
}

// ------------------------------------------------------------------------------------
constexpr int kRedWaves = 4;
constexpr int kRedBlock = kRedWaves * kWave;
template <typename T> struct RedCfg { static constexpr int kStageRows = 64; };
template <> struct RedCfg<float> { static constexpr int kStageRows = 32; };

// Block = (128 tokens, one (b, kv-head)); each wave keeps 32 tokens' key and value rows in
// registers as MFMA B operands (tokens -> lanes); the earlier tokens stream through LDS as
// the A operands (earlier token -> accumulator register).
template <typename T, int D>
__global__ __launch_bounds__(kRedBlock) void redundancy_kernel(StatsArgs a)
{
    constexpr int kStageRows = RedCfg<T>::kStageRows;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kStride = Tile<T, D>::kLdsStride;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kPerThread = kCpr * kStageRows / kRedBlock;

    __shared__ __attribute__((aligned(16))) char lds[2][kStageRows * kStride];
    __shared__ __attribute__((aligned(16))) float lds_rn[2][kStageRows];

    const int N = a.seq_len;
    const int bkv = blockIdx.y;
    const T* src[2] = {reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D,
                       reinterpret_cast<const T*>(a.v) + ((size_t)bkv * N) * D};
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    // heaviest blocks (latest tokens) first
    const int t_block0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * (kRedWaves * 32);
    const int ti = t_block0 + wave * 32 + col;               // this lane's token
    const bool t_ok = ti < N;

    frag_t bt[2][kFrags];
    float t_rn[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        float ss = 0.f;
#pragma unroll
        for (int f = 0; f < kFrags; ++f) {
            bt[s][f] = load_frag_or_zero(src[s], (size_t)(t_ok ? ti : 0) * Tile<T, D>::kRowBytes + f * 32 + half * 16, t_ok);
            ss += frag_sumsq<T>(bt[s][f]);
        }
        ss += __shfl_xor(ss, 32);
        t_rn[s] = inv_norm(ss);
    }

    float best = -INFINITY;
    const int c_end = min(N, t_block0 + kRedWaves * 32 - 1);  // earlier tokens the block can need
    // the next stage's rows are fetched into registers under the current stage's MFMAs
    frag_t pf[2][kPerThread];
    auto load_rows = [&](int c0) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int c = threadIdx.x + i * kRedBlock;
            const int ci = c0 + c / kCpr, cc = c % kCpr;
            const bool ok = ci < c_end;
#pragma unroll
            for (int s = 0; s < 2; ++s)
                pf[s][i] = load_frag_or_zero(src[s], ((size_t)(ok ? ci : 0) * kCpr + cc) * 16, ok);
        }
    };
    load_rows(0);
    for (int c0 = 0; c0 < c_end; c0 += kStageRows) {
        __syncthreads();                                   // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int c = threadIdx.x + i * kRedBlock;
            const int row = c / kCpr, cc = c % kCpr;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                *reinterpret_cast<frag_t*>(lds[s] + row * kStride + cc * 16) = pf[s][i];
                const float ss = group_sum<kCpr>(frag_sumsq<T>(pf[s][i]));
                if (cc == 0) lds_rn[s][row] = inv_norm(ss);
            }
        }
        __syncthreads();
        if (c0 + kStageRows < c_end) load_rows(c0 + kStageRows);   // block-uniform
#pragma unroll
        for (int rs = 0; rs < kStageRows / 32; ++rs) {
            const int cbase = c0 + rs * 32;
            if (cbase >= c_end || cbase >= t_block0 + wave * 32 + 31) continue;   // wave-uniform: nothing earlier here
            f32x16_t acc[2];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                acc[s] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < kFrags; ++f) {
                    const frag_t ac = *reinterpret_cast<const frag_t*>(lds[s] + (rs * 32 + col) * kStride + f * 32 + half * 16);
                    mma<T>(acc[s], ac, bt[s][f]);
                }
            }
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4_t rk = *reinterpret_cast<const f32x4_t*>(lds_rn[0] + rs * 32 + 8 * q4 + 4 * half);
                const f32x4_t rv = *reinterpret_cast<const f32x4_t*>(lds_rn[1] + rs * 32 + 8 * q4 + 4 * half);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ci = cbase + 8 * q4 + 4 * half + e;
                    const float r = ((acc[0][4 * q4 + e] * rk[e]) * t_rn[0]) * ((acc[1][4 * q4 + e] * rv[e]) * t_rn[1]);
                    if (ci < ti && r > best) best = r;       // strictly earlier tokens only
                }
            }
        }
    }
    best = fmaxf(best, __shfl_xor(best, 32));                // the other half-wave saw the other rows
    if (half == 0 && t_ok) a.best[(size_t)bkv * N + ti] = best;
}

__global__ __launch_bounds__(kStatBlock) void redundancy_count_kernel(StatsArgs a)
{
    __shared__ int total;
    const int N = a.seq_len;
    const float* best = a.best + (size_t)blockIdx.x * N;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    int mine = 0;
    for (int j = threadIdx.x; j < N; j += kStatBlock) mine += best[j] >= a.tau ? 1 : 0;   // Eq. 4: >=
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mine += __shfl_xor(mine, o);
    if (threadIdx.x % kWave == 0) atomicAdd(&total, mine);
    __syncthreads();
    if (threadIdx.x == 0) a.r_out[blockIdx.x] = (float)((double)total / (double)N);
}

hipError_t launch_sparsity(const StatsArgs& a, hipStream_t st)
{
    hipLaunchKernelGGL(sparsity_kernel, dim3(a.bkv), dim3(kStatBlock), 0, st, a);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_redundancy_t(const StatsArgs& a, hipStream_t st)
{
    const dim3 g((a.seq_len + kRedWaves * 32 - 1) / (kRedWaves * 32), a.bkv);
    hipLaunchKernelGGL((redundancy_kernel<T, D>), g, dim3(kRedBlock), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(redundancy_count_kernel, dim3(a.bkv), dim3(kStatBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_redundancy(const StatsArgs& a, bool f32, hipStream_t st)
{
    if (f32) return a.head_dim == 64 ? launch_redundancy_t<float, 64>(a, st) : launch_redundancy_t<float, 128>(a, st);
    return a.head_dim == 64 ? launch_redundancy_t<bf16_t, 64>(a, st) : launch_redundancy_t<bf16_t, 128>(a, st);
}

}  // namespace ems
