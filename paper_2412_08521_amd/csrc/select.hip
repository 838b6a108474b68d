// Global-Local score (Eq. 2), mean pooling and token partition (Sec. 4.2).
//
// Short sequences: one block per (batch, kv-head), keys in registers (select_reg_kernel).
// Long sequences: the O(N) part is spread over many blocks per head (see below).  Either way:
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

// Exclusive prefix sum of one int per thread over a block of kThreads (a multiple of 64, at most
// 1024); `total` gets the block's sum.  `sm` holds kThreads / 64 + 1 ints.  Every thread calls it.
template <int kThreads>
__device__ __forceinline__ int block_excl_scan(int v, int* sm, int& total)
{
    constexpr int kW = kThreads / kWave;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int incl = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(incl, o);
        if (lane >= o) incl += u;
    }
    __syncthreads();                                      // sm may still be read from an earlier call
    if (lane == kWave - 1) sm[wave] = incl;
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kW; ++w) { const int x = sm[w]; before += w < wave ? x : 0; tot += x; }
    total = tot;
    return before + incl - v;
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

// ------------------------------------------------------------------------------------
// Long sequences: every head is cut into chunks of kChunk positions, one block each, so that
// the whole chip works on the O(N) part; the exact ranking is then done by one block per head
// on a short list of candidates.  Four launches, in stream order:
//   A  select_sums_kernel     per-chunk sums of s_glo and s_loc (fixed-order trees)
//   B  select_keys_kernel     Eq. 2 with the head's factor (chunk sums added in a fixed tree),
//                             mean pooling, ranking keys written, and a histogram of the keys'
//                             12 leading bits per head (integer atomics: order-free)
//   C  select_gather_kernel   the leading-bit bin that holds the last rank wanted (N_imp +
//                             N_tbm): every key in that bin or above is a candidate; each chunk
//                             appends its candidates (key, position), in position order
//   D  select_finish_kernel   exact radix select of the two cut ranks over the candidates and
//                             ordered write of the two index sets
// The candidate list always contains every token of rank <= N_imp + N_tbm; with ties in the
// leading bits it is longer (in the extreme, all positions), which only costs time.
// ------------------------------------------------------------------------------------
constexpr int kChunk = 2048;          // positions per block in launches A-D
constexpr int kChunkBlock = 256;
constexpr int kPerThread = kChunk / kChunkBlock;
constexpr int kCoarseBits = 12, kCoarseBins = 1 << kCoarseBits;

__global__ __launch_bounds__(kChunkBlock) void select_sums_kernel(SelectArgs a)
{
    __shared__ float red[kChunkBlock / kWave][2];
    const int N = a.seq_len, head = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const float* glo = a.s_glo + (size_t)head * N;
    const float* loc = a.s_loc + (size_t)head * N;
    const int c0 = blk * kChunk;
    float sg = 0.f, sl = 0.f;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = c0 + i * kChunkBlock + tid;
        if (j < N) { sg += glo[j]; sl += loc[j]; }
    }
    sg = wave_sum(sg); sl = wave_sum(sl);
    if (tid % kWave == 0) { red[tid / kWave][0] = sg; red[tid / kWave][1] = sl; }
    __syncthreads();
    if (tid == 0) {
        float tg = 0.f, tl = 0.f;
        for (int w = 0; w < kChunkBlock / kWave; ++w) { tg += red[w][0]; tl += red[w][1]; }
        a.chunk_sums[((size_t)head * gridDim.x + blk) * 2 + 0] = tg;
        a.chunk_sums[((size_t)head * gridDim.x + blk) * 2 + 1] = tl;
    }
    // the head's histogram and list cursor start from zero (launches B and C add to them)
    if (blk == 0) {
        for (int b = tid; b < kCoarseBins; b += kChunkBlock) a.coarse_hist[(size_t)head * kCoarseBins + b] = 0;
        if (tid == 0) a.head_info[head] = 0;
    }
}

__global__ __launch_bounds__(kChunkBlock) void select_keys_kernel(SelectArgs a)
{
    extern __shared__ float comb_sm[];                     // chunk + halo on both sides
    __shared__ int hist[kCoarseBins];
    __shared__ float align_sm;
    const int N = a.seq_len, Nc = N - a.window, head = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const float* glo = a.s_glo + (size_t)head * N;
    const float* loc = a.s_loc + (size_t)head * N;
    for (int b = tid; b < kCoarseBins; b += kChunkBlock) hist[b] = 0;
    // all of the chunk's loads are in flight while the factor is being formed
    const int c0 = blk * kChunk;
    float g[kPerThread], l[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = c0 + i * kChunkBlock + tid;
        g[i] = j < N ? glo[j] : 0.f;
        l[i] = j < N ? loc[j] : 0.f;
    }
    // Eq. 2 factor: thread t adds the sums of chunks t, t + 256, ..., the wave adds its lanes with a
    // fixed butterfly, thread 0 adds the four waves in order -- the same tree in every block of the
    // head, so they all get the same factor bit for bit
    __shared__ float sums_sm[kChunkBlock / kWave][2];
    float tg = 0.f, tl = 0.f;
    for (int c = tid; c < (int)gridDim.x; c += kChunkBlock) {
        tg += a.chunk_sums[((size_t)head * gridDim.x + c) * 2 + 0];
        tl += a.chunk_sums[((size_t)head * gridDim.x + c) * 2 + 1];
    }
    tg = wave_sum(tg); tl = wave_sum(tl);
    if (tid % kWave == 0) { sums_sm[tid / kWave][0] = tg; sums_sm[tid / kWave][1] = tl; }
    __syncthreads();
    if (tid == 0) {
        float sg = 0.f, sl = 0.f;
#pragma unroll
        for (int w = 0; w < kChunkBlock / kWave; ++w) { sg += sums_sm[w][0]; sl += sums_sm[w][1]; }
        align_sm = (sl / (float)N) / (sg / (float)N);
    }
    __syncthreads();
    const float align = align_sm;
    const int half = (a.pool_kernel - 1) / 2;
    {
        for (int i = tid; i < 2 * half; i += kChunkBlock) {      // the halo: `half` positions on either side
            const int j = i < half ? c0 - half + i : c0 + kChunk + (i - half);
            comb_sm[i < half ? i : kChunk + i] = (j >= 0 && j < N) ? fmaxf(glo[j] * align, loc[j]) : 0.f;   // zero padding
        }
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int j = c0 + i * kChunkBlock + tid;
            comb_sm[half + i * kChunkBlock + tid] = j < N ? fmaxf(g[i] * align, l[i]) : 0.f;
        }
    }
    __syncthreads();
    const float div = (float)a.pool_kernel;
    float* pooled = a.pooled + (size_t)head * N;
    float* s_out = a.s_gl_opt ? a.s_gl_opt + (size_t)head * N : nullptr;
    // the window runs in the outer loop so that each step issues the thread's eight independent LDS
    // reads together (every element still adds its neighbours from left to right)
    float acc[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) acc[i] = 0.f;
    for (int t = 0; t <= 2 * half; ++t) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) acc[i] += comb_sm[i * kChunkBlock + tid + t];
    }
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = c0 + i * kChunkBlock + tid;
        const float v = acc[i] / div;
        if (j < N) { pooled[j] = v; if (s_out) s_out[j] = v; }
        hist_add(hist, (int)(order_key(v) >> (32 - kCoarseBits)), j < Nc);
    }
    __syncthreads();
    int* ghist = a.coarse_hist + (size_t)head * kCoarseBins;
    for (int b = tid; b < kCoarseBins; b += kChunkBlock)
        if (hist[b]) atomicAdd(&ghist[b], hist[b]);
}

// The lowest leading-bit bin a candidate may have: the bin that holds rank `want` counted from
// the top (every thread returns it).
__device__ __forceinline__ int coarse_cut_bin(const int* ghist, int want, int* scratch /* [kChunkBlock / 64 + 2] */)
{
    constexpr int kPer = kCoarseBins / kChunkBlock;        // bins per thread, taken from the top
    const int tid = threadIdx.x;
    int cnt[kPer], mine = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { cnt[i] = ghist[kCoarseBins - 1 - (tid * kPer + i)]; mine += cnt[i]; }
    int total;
    const int before = block_excl_scan<kChunkBlock>(mine, scratch, total);   // counts in the bins above this thread's
    int* answer = scratch + kChunkBlock / kWave + 1;
    if (tid == 0) *answer = 0;                             // fewer keys than wanted: everything is a candidate
    __syncthreads();
    if (before < want && before + mine >= want) {          // exactly one thread
        int cum = before;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            cum += cnt[i];
            if (cum >= want) { *answer = kCoarseBins - 1 - (tid * kPer + i); break; }
        }
    }
    __syncthreads();
    return *answer;
}

// Launch C: the candidates of a chunk, in position order, appended to the head's list.  A chunk
// reserves its stretch of the list with one integer atomic, so the stretches follow each other
// in whatever order the blocks arrive; where each chunk's stretch starts and how long it is is
// recorded, and launch D reads the list chunk by chunk -- its result does not depend on the
// arrival order.
__global__ __launch_bounds__(kChunkBlock) void select_gather_kernel(SelectArgs a)
{
    __shared__ int scratch[kChunkBlock / kWave + 2];
    __shared__ int base_sm;
    const int N = a.seq_len, Nc = N - a.window, head = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    // the chunk's keys are requested before the histogram is scanned (independent round trips)
    const int c0 = blk * kChunk;
    float pv[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = c0 + tid * kPerThread + i;
        pv[i] = j < Nc ? (a.pooled + (size_t)head * N)[j] : 0.f;
    }
    const int cut_bin = coarse_cut_bin(a.coarse_hist + (size_t)head * kCoarseBins, a.n_imp + a.n_tbm, scratch);
    uint32_t key[kPerThread];
    int n = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = c0 + tid * kPerThread + i;
        key[i] = j < Nc ? order_key(pv[i]) : 0u;
        n += (j < Nc && (int)(key[i] >> (32 - kCoarseBits)) >= cut_bin) ? 1 : 0;
    }
    int total;
    const int before = block_excl_scan<kChunkBlock>(n, scratch, total);
    if (tid == 0) {
        base_sm = atomicAdd(&a.head_info[head], total);
        a.chunk_count[((size_t)head * gridDim.x + blk) * 2 + 0] = base_sm;
        a.chunk_count[((size_t)head * gridDim.x + blk) * 2 + 1] = total;
    }
    __syncthreads();
    int at = base_sm + before;
    uint32_t* ckey = a.cand_key + (size_t)head * N;
    int32_t* cpos = a.cand_pos + (size_t)head * N;
    const int j0 = c0 + tid * kPerThread;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int j = j0 + i;
        if (j < Nc && (int)(key[i] >> (32 - kCoarseBits)) >= cut_bin) { ckey[at] = key[i]; cpos[at] = j; ++at; }
    }
}

// Launch D: exact two-cut selection over a head's candidate list (keys already in integer order
// form): steps 3 and 4 of the header comment.  The list is a sequence of per-chunk stretches in
// arbitrary order; position order is chunk order, then order inside the stretch.
constexpr int kMaxChunks = (1 << 22) / kChunk;   // the interface limits seq_len to 2^22
__global__ __launch_bounds__(kSelBlock) void select_finish_kernel(SelectArgs a)
{
    __shared__ int hist[2][256];
    __shared__ int suffix[2][257];
    __shared__ int scan_sm[kSelWaves][2];
    __shared__ int wave_tot[8];
    __shared__ uint32_t sel_prefix[2];
    __shared__ int sel_rem[2];
    __shared__ int ch_first[kMaxChunks + 1];     // rank (in position order) of a chunk's first candidate
    __shared__ int ch_at[kMaxChunks];            // where its stretch starts in the list
    __shared__ int scan17[kSelWaves + 1];

    const int N = a.seq_len;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const uint32_t* ckey = a.cand_key + (size_t)blockIdx.x * N;
    const int32_t* cpos = a.cand_pos + (size_t)blockIdx.x * N;
    const int n_chunks = a.n_chunks;
    int M = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += kSelBlock) {     // exclusive scan of the chunk lengths, in chunk order
        const int c = c0 + tid;
        const int len = c < n_chunks ? a.chunk_count[((size_t)blockIdx.x * n_chunks + c) * 2 + 1] : 0;
        int total;
        const int before = block_excl_scan<kSelBlock>(len, scan17, total);
        if (c < n_chunks) { ch_first[c] = M + before; ch_at[c] = a.chunk_count[((size_t)blockIdx.x * n_chunks + c) * 2]; }
        M += total;
    }
    if (tid == 0) ch_first[n_chunks] = M;
    __syncthreads();
    // list index of the candidate of rank j in position order
    auto at_rank = [&](int j) {
        int lo = 0, hi = n_chunks;                         // ch_first[lo] <= j < ch_first[hi]
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (ch_first[mid] <= j) lo = mid; else hi = mid; }
        return ch_at[lo] + (j - ch_first[lo]);
    };

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
        for (int j0 = tid; j0 < M; j0 += kSelBlock * kSelUnroll) {
            uint32_t key[kSelUnroll];
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const int j = j0 + u * kSelBlock;
                key[u] = j < M ? ckey[j] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kSelUnroll; ++u) {
                const bool ok = j0 + u * kSelBlock < M;
                if (__ballot(ok) == 0ull) continue;                  // wave-uniform
                const uint32_t hi = shift == 24 ? 0u : (key[u] >> (shift + 8));
                const int digit = (key[u] >> shift) & 255;
                hist_add(hist[0], digit, ok && (shift == 24 || hi == p0));
                if (!same_prefix) hist_add(hist[1], digit, ok && hi == p1);
            }
        }
        __syncthreads();
        if (same_prefix && tid < 256) hist[1][tid] = hist[0][tid];   // one count serves both cuts
        __syncthreads();
        // suffix[t][d] = number of matching keys with digit >= d
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

    // ---- 4. ordered classification: rank = #greater + #equal at lower positions.  Every wave
    // owns a contiguous range of the list and walks it 64 at a time; ordinals inside a step come
    // from ballots, across steps from running counters, across waves from a scan over the wave totals.
    const int per_wave = ((M + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int w0 = min(wave * per_wave, M), w1 = min(w0 + per_wave, M);
    const unsigned long long below = (1ull << lane) - 1ull;
    auto wave_prefix = [&](int mine, int& before) {                 // exclusive scan over waves
        __syncthreads();
        if (lane == 0) scan_sm[wave][0] = mine;
        __syncthreads();
        before = 0;
        for (int w = 0; w < wave; ++w) before += scan_sm[w][0];
    };
    int eq1 = 0, eq2 = 0;
    for (int j = w0 + lane; j < w1 + lane; j += kWave) {
        const bool ok = j < w1;
        const uint32_t key = ok ? ckey[at_rank(j)] : 0u;
        eq1 += __popcll(__ballot(ok && key == T1));
        eq2 += __popcll(__ballot(ok && key == T2));
    }
    int o1, o2;
    wave_prefix(eq1, o1);
    wave_prefix(eq2, o2);
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
    int c_imp = 0, c_tbm = 0;
    {
        int r1 = o1, r2 = o2;
        for (int j = w0 + lane; j < w1 + lane; j += kWave) {
            const bool ok = j < w1;
            const uint32_t key = ok ? ckey[at_rank(j)] : 0u;
            bool ii, tt;
            classify(key, ok, r1, r2, ii, tt);
            c_imp += __popcll(__ballot(ii));
            c_tbm += __popcll(__ballot(tt));
        }
    }
    int bi, bt;
    wave_prefix(c_imp, bi);
    wave_prefix(c_tbm, bt);
    int32_t* imp = a.imp_idx + (size_t)blockIdx.x * a.n_imp;
    int32_t* tbm = a.tbm_idx ? a.tbm_idx + (size_t)blockIdx.x * a.n_tbm : nullptr;
    {
        int r1 = o1, r2 = o2;
        for (int j = w0 + lane; j < w1 + lane; j += kWave) {
            const bool ok = j < w1;
            const int jl = ok ? at_rank(j) : 0;
            const uint32_t key = ok ? ckey[jl] : 0u;
            bool ii, tt;
            classify(key, ok, r1, r2, ii, tt);
            const unsigned long long mi = __ballot(ii), mt = __ballot(tt);
            if (ii) { const int at = bi + __popcll(mi & below); if (at < a.n_imp) imp[at] = cpos[jl]; }
            if (tt && tbm) { const int at = bt + __popcll(mt & below); if (at < a.n_tbm) tbm[at] = cpos[jl]; }
            bi += __popcll(mi); bt += __popcll(mt);
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
    const dim3 grid((unsigned)select_chunks(a.seq_len), (unsigned)a.bkv);
    const size_t lds = sizeof(float) * (size_t)(kChunk + a.pool_kernel - 1);
    hipLaunchKernelGGL(select_sums_kernel, grid, dim3(kChunkBlock), 0, st, a);
    hipLaunchKernelGGL(select_keys_kernel, grid, dim3(kChunkBlock), lds, st, a);
    hipLaunchKernelGGL(select_gather_kernel, grid, dim3(kChunkBlock), 0, st, a);
    hipLaunchKernelGGL(select_finish_kernel, dim3((unsigned)a.bkv), dim3(kSelBlock), 0, st, a);
    return hipGetLastError();
}

int select_chunks(int seq_len) { return (seq_len + kChunk - 1) / kChunk; }
int select_coarse_bins() { return kCoarseBins; }

}  // namespace ems
