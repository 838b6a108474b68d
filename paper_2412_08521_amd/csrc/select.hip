// Global-Local score (Eq. 2), mean pooling and token partition (Sec. 4.2).
//
// One block per (batch, kv-head).  The block
//   1. sums s_glo and s_loc (fixed-order tree) to get the mean-alignment factor of Eq. 2,
//   2. forms s = max(s_glo * factor, s_loc) and its zero-padded mean pool, written as the
//      ranking key of every position,
//   3. finds, by an 8-bit-digit radix select over the order-preserving integer image of
//      the keys, the key value at rank N_imp and at rank N_imp + N_tbm among the
//      candidates (all positions before the local window), together with how many
//      elements equal to that value still belong above the cut,
//   4. walks the candidates in position order and writes the important / to-be-merged
//      positions ascending; equal keys rank by lower position first.
// Integer work only after step 2, so the index sets are a pure function of the keys.
#include "ems_common.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / kWave;

// Monotone map float -> uint32 (larger float <=> larger integer), also for negatives.
__device__ __forceinline__ uint32_t order_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Exclusive prefix sums over the block (thread order) of two integers; also the totals.
__device__ __forceinline__ void block_scan2(int a, int b, int& ea, int& eb, int& ta, int& tb,
                                            int (*sm)[2])
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int ia = a, ib = b;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int ua = __shfl_up(ia, o), ub = __shfl_up(ib, o);
        if (lane >= o) { ia += ua; ib += ub; }
    }
    __syncthreads();
    if (lane == kWave - 1) { sm[wave][0] = ia; sm[wave][1] = ib; }
    __syncthreads();
    int wa = 0, wb = 0, sa = 0, sb = 0;
    for (int w = 0; w < kSelWaves; ++w) {
        const int xa = sm[w][0], xb = sm[w][1];
        if (w < wave) { wa += xa; wb += xb; }
        sa += xa; sb += xb;
    }
    ea = wa + ia - a; eb = wb + ib - b; ta = sa; tb = sb;
}

__global__ __launch_bounds__(kSelBlock) void select_kernel(SelectArgs a)
{
    __shared__ float red[kSelWaves][2];
    __shared__ int hist[2][256];
    __shared__ int suffix[2][257];
    __shared__ int scan_sm[kSelWaves][2];
    __shared__ int wave_tot[8];
    __shared__ uint32_t sel_prefix[2];
    __shared__ int sel_rem[2];

    const int N = a.seq_len, Nc = N - a.window;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const float* glo = a.s_glo + (size_t)blockIdx.x * N;
    const float* loc = a.s_loc + (size_t)blockIdx.x * N;
    float* pooled = a.pooled + (size_t)blockIdx.x * N;
    float* s_out = a.s_gl_opt ? a.s_gl_opt + (size_t)blockIdx.x * N : nullptr;

    // ---- 1. Eq. 2 alignment factor (sum(s_loc)/N) / (sum(s_glo)/N)
    float sg = 0.f, sl = 0.f;
    for (int j = tid; j < N; j += kSelBlock) { sg += glo[j]; sl += loc[j]; }
    sg = wave_sum(sg); sl = wave_sum(sl);
    if (lane == 0) { red[wave][0] = sg; red[wave][1] = sl; }
    __syncthreads();
    float tot_g = 0.f, tot_l = 0.f;
    for (int w = 0; w < kSelWaves; ++w) { tot_g += red[w][0]; tot_l += red[w][1]; }
    const float align = (tot_l / (float)N) / (tot_g / (float)N);

    // ---- 2. element-wise max and mean pooling (zero padding, divisor = kernel width)
    const int half = (a.pool_kernel - 1) / 2;
    const float inv_div = (float)a.pool_kernel;
    for (int j = tid; j < N; j += kSelBlock) {
        float acc = 0.f;
        for (int t = -half; t <= half; ++t) {
            const int jj = j + t;
            if (jj >= 0 && jj < N) acc += fmaxf(glo[jj] * align, loc[jj]);
        }
        const float v = acc / inv_div;
        pooled[j] = v;
        if (s_out) s_out[j] = v;
    }
    __syncthreads();   // this block's global writes are visible to the whole block

    // ---- 3. radix select of two ranks (1-based, counted from the largest key)
    if (tid < 2) {
        sel_prefix[tid] = 0u;
        sel_rem[tid] = tid == 0 ? a.n_imp : a.n_imp + a.n_tbm;
    }
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 512) hist[tid >> 8][tid & 255] = 0;
        __syncthreads();
        const uint32_t p0 = sel_prefix[0], p1 = sel_prefix[1];
        for (int j = tid; j < Nc; j += kSelBlock) {
            const uint32_t key = order_key(pooled[j]);
            const uint32_t hi = shift == 24 ? 0u : (key >> (shift + 8));
            const int digit = (key >> shift) & 255;
            if (shift == 24 || hi == p0) atomicAdd(&hist[0][digit], 1);
            if (shift == 24 || hi == p1) atomicAdd(&hist[1][digit], 1);
        }
        __syncthreads();
        // suffix[t][d] = number of matching keys with digit >= d: an inclusive scan over
        // the digits taken from 255 downwards, 256 threads per target (4 waves each).
        int incl = 0;
        if (tid < 512) {
            incl = hist[tid >> 8][255 - (tid & 255)];
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int u = __shfl_up(incl, o);
                if (lane >= o) incl += u;
            }
            if (lane == kWave - 1) wave_tot[wave] = incl;
        }
        __syncthreads();
        if (tid < 512) {
            const int t = tid >> 8;
            for (int w = t * 4; w < wave; ++w) incl += wave_tot[w];
            suffix[t][255 - (tid & 255)] = incl;
            if ((tid & 255) == 0) suffix[t][256] = 0;
        }
        __syncthreads();
        bool mine = false;
        uint32_t new_prefix = 0u;
        int new_rem = 0;
        if (tid < 512) {
            const int t = tid >> 8, d = tid & 255;
            const int rem = sel_rem[t];
            mine = suffix[t][d] >= rem && suffix[t][d + 1] < rem;
            new_prefix = (sel_prefix[t] << 8) | (uint32_t)d;
            new_rem = rem - suffix[t][d + 1];
        }
        __syncthreads();
        if (mine) { sel_prefix[tid >> 8] = new_prefix; sel_rem[tid >> 8] = new_rem; }
        __syncthreads();
    }
    const uint32_t T1 = sel_prefix[0], T2 = sel_prefix[1];
    const int need1 = sel_rem[0];                 // keys equal to T1 that rank inside N_imp
    const int k1 = a.n_imp, k2 = a.n_imp + a.n_tbm;
    const int G1 = k1 - need1;                    // keys greater than T1
    const int G2 = k2 - sel_rem[1];               // keys greater than T2

    // ---- 4. ordered classification: rank = #greater + #equal at lower positions
    const int per = (Nc + kSelBlock - 1) / kSelBlock;
    const int j0 = min(tid * per, Nc), j1 = min(j0 + per, Nc);
    int eq1 = 0, eq2 = 0;
    for (int j = j0; j < j1; ++j) {
        const uint32_t key = order_key(pooled[j]);
        eq1 += key == T1;
        eq2 += key == T2;
    }
    int o1, o2, t1, t2;
    block_scan2(eq1, eq2, o1, o2, t1, t2, scan_sm);
    int n_imp = 0, n_tbm = 0;
    {
        int r1 = o1, r2 = o2;
        for (int j = j0; j < j1; ++j) {
            const uint32_t key = order_key(pooled[j]);
            int rank;
            if (key == T1) rank = G1 + r1++;
            else if (key == T2) rank = G2 + r2++;
            else rank = key > T1 ? 0 : (key > T2 ? k1 : k2);
            n_imp += rank < k1;
            n_tbm += rank >= k1 && rank < k2;
        }
    }
    int bi, bt, ti, tt;
    block_scan2(n_imp, n_tbm, bi, bt, ti, tt, scan_sm);
    int32_t* imp = a.imp_idx + (size_t)blockIdx.x * a.n_imp;
    int32_t* tbm = a.tbm_idx ? a.tbm_idx + (size_t)blockIdx.x * a.n_tbm : nullptr;
    {
        int r1 = o1, r2 = o2;
        for (int j = j0; j < j1; ++j) {
            const uint32_t key = order_key(pooled[j]);
            int rank;
            if (key == T1) rank = G1 + r1++;
            else if (key == T2) rank = G2 + r2++;
            else rank = key > T1 ? 0 : (key > T2 ? k1 : k2);
            if (rank < k1) { if (bi < a.n_imp) imp[bi] = j; ++bi; }
            else if (rank < k2) { if (tbm && bt < a.n_tbm) tbm[bt] = j; ++bt; }
        }
    }
}

hipError_t launch_select(const SelectArgs& a, hipStream_t st)
{
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)a.bkv), dim3(kSelBlock), 0, st, a);
    return hipGetLastError();
}

}  // namespace ems
