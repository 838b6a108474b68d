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
constexpr int kSelUnroll = 8;     // keys in flight per thread in the loops that re-read them from memory

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

// One histogram update per lane (if `on`).  Scores share their leading digits, so most
// lanes of a wave hit the same bin: the lanes that agree with the first active lane are
// counted with one ballot and one atomic, the others fall back to their own atomic.
__device__ __forceinline__ void hist_add(int* hist, int digit, bool on)
{
    const unsigned long long active = __ballot(on);
    if (active == 0ull) return;                                   // wave-uniform
    const int leader = __ffsll((long long)active) - 1;
    const int d0 = __shfl(digit, leader);
    const unsigned long long same = __ballot(on && digit == d0);
    if ((int)(threadIdx.x % kWave) == leader) atomicAdd(&hist[d0], __popcll(same));
    if (on && digit != d0) atomicAdd(&hist[digit], 1);
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

    // ---- 2. element-wise max, staged through the workspace, then mean pooling (zero padding,
    // divisor = kernel width)
    float* comb = a.comb + (size_t)blockIdx.x * N;
    for (int j = tid; j < N; j += kSelBlock) comb[j] = fmaxf(glo[j] * align, loc[j]);
    __syncthreads();   // this block's global writes are visible to the whole block
    const int half = (a.pool_kernel - 1) / 2;
    const float inv_div = (float)a.pool_kernel;
    for (int j = tid; j < N; j += kSelBlock) {
        float acc = 0.f;
        for (int t = -half; t <= half; ++t) {
            const int jj = j + t;
            if (jj >= 0 && jj < N) acc += comb[jj];
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
        const bool same_prefix = shift == 24 || p0 == p1;
        // eight keys in flight per thread: the loop is bound by load latency otherwise
        for (int j0 = tid; j0 < Nc; j0 += kSelBlock * kSelUnroll) {
            uint32_t key[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const int j = j0 + u * kSelBlock;
                key[u] = j < Nc ? order_key(pooled[j]) : 0u;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const bool ok = j0 + u * kSelBlock < Nc;
                const uint32_t hi = shift == 24 ? 0u : (key[u] >> (shift + 8));
                const int digit = (key[u] >> shift) & 255;
                hist_add(hist[0], digit, ok && (shift == 24 || hi == p0));
                if (!same_prefix) hist_add(hist[1], digit, ok && hi == p1);
            }
        }
        __syncthreads();
        if (same_prefix && tid < 256) hist[1][tid] = hist[0][tid];   // one count serves both cuts
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

    // ---- 4. ordered classification: rank = #greater + #equal at lower positions.
    // Every wave owns a contiguous range of positions and walks it 64 at a time (coalesced);
    // ordinals inside a step come from ballots, across steps from running counters, across
    // waves from a scan over the 16 wave totals.
    const int per_wave = ((Nc + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int w0 = min(wave * per_wave, Nc), w1 = min(w0 + per_wave, Nc);
    const unsigned long long below = (1ull << lane) - 1ull;
    auto wave_prefix = [&](int mine, int& before, int& total) {     // exclusive scan over waves
        __syncthreads();
        if (lane == 0) scan_sm[wave][0] = mine;
        __syncthreads();
        before = 0; total = 0;
        for (int w = 0; w < kSelWaves; ++w) { const int x = scan_sm[w][0]; if (w < wave) before += x; total += x; }
    };
    // pass A: how many keys equal to each cut value does every wave hold
    int eq1 = 0, eq2 = 0;
    for (int j0 = w0 + lane; j0 < w1 + lane; j0 += kWave * kSelUnroll) {
        uint32_t key[kSelUnroll];
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
            const int j = j0 + u * kWave;
            key[u] = j < w1 ? order_key(pooled[j]) : 0u;
        }
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
            const bool ok = j0 + u * kWave < w1;
            eq1 += __popcll(__ballot(ok && key[u] == T1));
            eq2 += __popcll(__ballot(ok && key[u] == T2));
        }
    }
    int o1, o2, tot;
    wave_prefix(eq1, o1, tot);
    wave_prefix(eq2, o2, tot);
    auto classify = [&](uint32_t key, bool ok, int& r1, int& r2, bool& is_imp, bool& is_tbm) {
        const unsigned long long m1 = __ballot(ok && key == T1), m2 = __ballot(ok && key == T2);
        int rank;
        if (key == T1) rank = G1 + r1 + __popcll(m1 & below);
        else if (key == T2) rank = G2 + r2 + __popcll(m2 & below);
        else rank = key > T1 ? 0 : (key > T2 ? k1 : k2);
        r1 += __popcll(m1); r2 += __popcll(m2);
        is_imp = ok && rank < k1;
        is_tbm = ok && rank >= k1 && rank < k2;
    };
    // pass B: how many important / to-be-merged tokens does every wave hold
    int c_imp = 0, c_tbm = 0;
    {
        int r1 = o1, r2 = o2;
        for (int j0 = w0 + lane; j0 < w1 + lane; j0 += kWave * kSelUnroll) {
            uint32_t key[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const int j = j0 + u * kWave;
                key[u] = j < w1 ? order_key(pooled[j]) : 0u;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const bool ok = j0 + u * kWave < w1;
                if (__ballot(ok && key[u] >= T2) == 0ull) continue;   // wave-uniform: nothing to rank here
                bool ii, tt;
                classify(key[u], ok, r1, r2, ii, tt);
                c_imp += __popcll(__ballot(ii));
                c_tbm += __popcll(__ballot(tt));
            }
        }
    }
    int bi, bt;
    wave_prefix(c_imp, bi, tot);
    wave_prefix(c_tbm, bt, tot);
    // pass C: write the positions, ascending
    int32_t* imp = a.imp_idx + (size_t)blockIdx.x * a.n_imp;
    int32_t* tbm = a.tbm_idx ? a.tbm_idx + (size_t)blockIdx.x * a.n_tbm : nullptr;
    {
        int r1 = o1, r2 = o2;
        for (int j0 = w0 + lane; j0 < w1 + lane; j0 += kWave * kSelUnroll) {
            uint32_t key[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const int j = j0 + u * kWave;
                key[u] = j < w1 ? order_key(pooled[j]) : 0u;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const int j = j0 + u * kWave;
                const bool ok = j < w1;
                if (__ballot(ok && key[u] >= T2) == 0ull) continue;   // wave-uniform
                bool ii, tt;
                classify(key[u], ok, r1, r2, ii, tt);
                const unsigned long long mi = __ballot(ii), mt = __ballot(tt);
                if (ii) { const int at = bi + __popcll(mi & below); if (at < a.n_imp) imp[at] = j; }
                if (tt && tbm) { const int at = bt + __popcll(mt & below); if (at < a.n_tbm) tbm[at] = j; }
                bi += __popcll(mi); bt += __popcll(mt);
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// Same computation with the ranking keys held in registers.  Wave w owns the positions
// [w * 64 * kItems, (w + 1) * 64 * kItems); lane l holds positions base + i * 64 + l, so
// every load and store is coalesced and, after the keys are formed, nothing depends on
// memory latency any more.  Used when the sequence fits (N <= 1024 * kItems).
// ------------------------------------------------------------------------------------
template <int kItems>
__global__ __launch_bounds__(kSelBlock) void select_reg_kernel(SelectArgs a)
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
    float* comb = a.pooled + (size_t)blockIdx.x * N;      // Eq. 2 vector, before pooling
    float* s_out = a.s_gl_opt ? a.s_gl_opt + (size_t)blockIdx.x * N : nullptr;
    const int base = wave * kWave * kItems + lane;        // position of item i: base + 64 i

    // ---- 1. Eq. 2 alignment factor (sum(s_loc)/N) / (sum(s_glo)/N)
    float g[kItems], l[kItems];
    float sg = 0.f, sl = 0.f;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int j = base + i * kWave;
        g[i] = j < N ? glo[j] : 0.f;
        l[i] = j < N ? loc[j] : 0.f;
        sg += g[i]; sl += l[i];
    }
    sg = wave_sum(sg); sl = wave_sum(sl);
    if (lane == 0) { red[wave][0] = sg; red[wave][1] = sl; }
    __syncthreads();
    float tot_g = 0.f, tot_l = 0.f;
    for (int w = 0; w < kSelWaves; ++w) { tot_g += red[w][0]; tot_l += red[w][1]; }
    const float align = (tot_l / (float)N) / (tot_g / (float)N);

    // ---- 2. element-wise max, staged through the workspace so that the pooling window
    // can reach into the neighbouring lanes' and waves' positions
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int j = base + i * kWave;
        if (j < N) comb[j] = fmaxf(g[i] * align, l[i]);
    }
    __syncthreads();   // the block's own global writes are visible to the whole block
    const int half = (a.pool_kernel - 1) / 2;
    const float div = (float)a.pool_kernel;
    uint32_t key[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int j = base + i * kWave;
        float acc = 0.f;
        if (half <= 3) {
            // the usual window (width <= 7): independent, unconditional loads
            float nb[7];
#pragma unroll
            for (int t = -3; t <= 3; ++t) nb[t + 3] = comb[min(max(j + t, 0), N - 1)];
#pragma unroll
            for (int t = -3; t <= 3; ++t)
                acc += (t >= -half && t <= half && j + t >= 0 && j + t < N) ? nb[t + 3] : 0.f;
        } else {
            for (int t = -half; t <= half; ++t) {
                const int jj = j + t;
                if (jj >= 0 && jj < N) acc += comb[jj];
            }
        }
        const float v = acc / div;
        key[i] = order_key(v);
        if (s_out && j < N) s_out[j] = v;
    }

    // ---- 3. radix select of two ranks (1-based, counted from the largest key)
    if (tid < 2) {
        sel_prefix[tid] = 0u;
        sel_rem[tid] = tid == 0 ? a.n_imp : a.n_imp + a.n_tbm;
    }
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 512) hist[tid >> 8][tid & 255] = 0;
        __syncthreads();
        const uint32_t p0 = sel_prefix[0], p1 = sel_prefix[1];
        const bool same_prefix = shift == 24 || p0 == p1;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const bool cand = base + i * kWave < Nc;
            const uint32_t hi = shift == 24 ? 0u : (key[i] >> (shift + 8));
            const int digit = (key[i] >> shift) & 255;
            hist_add(hist[0], digit, cand && (shift == 24 || hi == p0));
            if (!same_prefix) hist_add(hist[1], digit, cand && hi == p1);
        }
        __syncthreads();
        if (same_prefix && tid < 256) hist[1][tid] = hist[0][tid];   // one count serves both cuts
        __syncthreads();
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
    const int k1 = a.n_imp, k2 = a.n_imp + a.n_tbm;
    const int G1 = k1 - sel_rem[0];               // keys greater than T1
    const int G2 = k2 - sel_rem[1];               // keys greater than T2

    // ---- 4. ordered classification: rank = #greater + #equal at lower positions; position
    // order inside a wave is (item, lane), across waves the wave number
    auto below_count = [&](unsigned long long m) {                 // set bits of m below this lane
        return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    };
    auto wave_prefix = [&](int mine_, int& before) {               // exclusive scan over waves
        __syncthreads();
        if (lane == 0) scan_sm[wave][0] = mine_;
        __syncthreads();
        before = 0;
        for (int w = 0; w < wave; ++w) before += scan_sm[w][0];
    };
    int eq1 = 0, eq2 = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const bool cand = base + i * kWave < Nc;
        eq1 += __popcll(__ballot(cand && key[i] == T1));
        eq2 += __popcll(__ballot(cand && key[i] == T2));
    }
    int r1, r2;
    wave_prefix(eq1, r1);
    wave_prefix(eq2, r2);
    unsigned imp_mask = 0u, tbm_mask = 0u;        // bit i: item i; kItems <= 32
    int c_imp = 0, c_tbm = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const bool cand = base + i * kWave < Nc;
        // almost every (wave, item) slice lies entirely below the second cut: nothing to rank
        if (__ballot(cand && key[i] >= T2) == 0ull) continue;         // wave-uniform
        const unsigned long long m1 = __ballot(cand && key[i] == T1), m2 = __ballot(cand && key[i] == T2);
        int rank;
        if (key[i] == T1) rank = G1 + r1 + below_count(m1);
        else if (key[i] == T2) rank = G2 + r2 + below_count(m2);
        else rank = key[i] > T1 ? 0 : (key[i] > T2 ? k1 : k2);
        r1 += __popcll(m1); r2 += __popcll(m2);
        const bool ii = cand && rank < k1, tt = cand && rank >= k1 && rank < k2;
        if (ii) imp_mask |= 1u << i;
        if (tt) tbm_mask |= 1u << i;
        c_imp += __popcll(__ballot(ii));
        c_tbm += __popcll(__ballot(tt));
    }
    int bi, bt;
    wave_prefix(c_imp, bi);
    wave_prefix(c_tbm, bt);
    int32_t* imp = a.imp_idx + (size_t)blockIdx.x * a.n_imp;
    int32_t* tbm = a.tbm_idx ? a.tbm_idx + (size_t)blockIdx.x * a.n_tbm : nullptr;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const bool ii = (imp_mask >> i) & 1u, tt = (tbm_mask >> i) & 1u;
        if (__ballot(ii || tt) == 0ull) continue;                        // wave-uniform
        const unsigned long long mi = __ballot(ii), mt = __ballot(tt);
        if (ii) { const int at = bi + below_count(mi); if (at < a.n_imp) imp[at] = base + i * kWave; }
        if (tt && tbm) { const int at = bt + below_count(mt); if (at < a.n_tbm) tbm[at] = base + i * kWave; }
        bi += __popcll(mi); bt += __popcll(mt);
    }
}

template <int kItems>
static hipError_t launch_select_reg(const SelectArgs& a, hipStream_t st)
{
    hipLaunchKernelGGL(select_reg_kernel<kItems>, dim3((unsigned)a.bkv), dim3(kSelBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_select(const SelectArgs& a, hipStream_t st)
{
    if (a.seq_len <= kSelBlock * 2) return launch_select_reg<2>(a, st);
    if (a.seq_len <= kSelBlock * 8) return launch_select_reg<8>(a, st);
    if (a.seq_len <= kSelBlock * 32) return launch_select_reg<32>(a, st);
    hipLaunchKernelGGL(select_kernel, dim3((unsigned)a.bkv), dim3(kSelBlock), 0, st, a);
    return hipGetLastError();
}

}  // namespace ems
