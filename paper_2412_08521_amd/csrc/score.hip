// Global / Local accumulated attention scores (Sec. 3.2) on gfx950 matrix cores.
//
// Two passes over the causal logits S = scale * Q K^T, neither of which stores an N x N
// matrix (App. A, "Global-Local Score Efficiency Discussion"):
//   pass 1 (query-stationary)  per row i: lse2_i = log2 sum_{j<=i} 2^(c S_ij), c = log2(e)
//   pass 2 (key-stationary)    per key j: sum over rows i >= j of 2^(c S_ij - lse2_i),
//                              once over all rows (global) and once over the last
//                              `window` rows (local), summed over the q-heads of a group.
// Both passes orient the MFMA so that the index being reduced over lives in the
// accumulator's registers and the index being kept lives in the lanes: reductions are
// in-register adds plus one exchange between the two half-waves, no atomics anywhere.
#include "ems_common.h"
#include "ems_kernels.h"

namespace ems {

constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWavesPerBlock * kWave;
// Per element type: 32-wide subtiles of the stationary operand a wave keeps in registers,
// and rows of the streamed operand staged in LDS per step (sized so that two stages of
// the widest row stay well inside the static LDS limit).
template <typename T> struct Sub { static constexpr int kSub = 2; static constexpr int kStageRows = 64; };
template <> struct Sub<float> { static constexpr int kSub = 1; static constexpr int kStageRows = 32; };

// Stage kStageRows rows (row0 onwards of a [n_rows, D] matrix) into registers; rows past
// the end read as zeros.
template <typename T, int D> struct StageRegs {
    static constexpr int kPerThread = Tile<T, D>::kChunksPerRow * Sub<T>::kStageRows / kBlock;
    frag_t r[kPerThread];
};

template <typename T, int D>
__device__ __forceinline__ void stage_load(StageRegs<T, D>& regs, const T* base, int row0, int n_rows)
{
    constexpr int kStageRows = Sub<T>::kStageRows;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kPerThread = kCpr * kStageRows / kBlock;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int c = threadIdx.x + i * kBlock;
        const int row = c / kCpr, col = c % kCpr;
        const int grow = row0 + row;
        regs.r[i] = load_frag_or_zero(base, ((size_t)grow * kCpr + col) * 16, grow < n_rows);
    }
}

template <typename T, int D>
__device__ __forceinline__ void stage_store(char* lds, const StageRegs<T, D>& regs)
{
    constexpr int kStageRows = Sub<T>::kStageRows;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kPerThread = kCpr * kStageRows / kBlock;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int c = threadIdx.x + i * kBlock;
        const int row = c / kCpr, col = c % kCpr;
        *reinterpret_cast<frag_t*>(lds + row * Tile<T, D>::kLdsStride + col * 16) = regs.r[i];
    }
}

// ------------------------------------------------------------------------------------
// Pass 1.  Block = (b, q-head, tile of 4 * 32 * kSub query rows).  Each wave keeps its
// queries in registers as the MFMA B operand (queries -> lanes) and streams key tiles
// through LDS as the A operand (keys -> accumulator registers), so the running row
// maximum and row sum of the online softmax are per-lane scalars.
// ------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void score_pass1_kernel(ScoreArgs a)
{
    constexpr int kSub = Sub<T>::kSub;
    constexpr int kStageRows = Sub<T>::kStageRows;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kStride = Tile<T, D>::kLdsStride;
    constexpr int kRowsPerBlock = kWavesPerBlock * 32 * kSub;

    __shared__ __attribute__((aligned(16))) char lds[2][kStageRows * kStride];

    const int N = a.seq_len;
    const int n_row_tiles = (N + kRowsPerBlock - 1) / kRowsPerBlock;
    const int G = a.q_heads / a.kv_heads;
    // (b, kv-head) outermost so that blocks in flight share one K; heaviest row tiles first.
    int bid = blockIdx.x;
    const int g = bid % G; bid /= G;
    const int rt = n_row_tiles - 1 - (bid % n_row_tiles); bid /= n_row_tiles;
    const int bkv = bid;                          // b * kv_heads + kv
    const int b = bkv / a.kv_heads, kvh = bkv % a.kv_heads;
    const int h = kvh * G + g;

    const T* Q = reinterpret_cast<const T*>(a.q) + ((size_t)(b * a.q_heads + h) * N) * D;
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    const int q0 = rt * kRowsPerBlock + wave * 32 * kSub;

    frag_t bq[kSub][kFrags];
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const int qi = q0 + s * 32 + col;
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            bq[s][f] = load_frag_or_zero(Q, (size_t)qi * Tile<T, D>::kRowBytes + f * 32 + half * 16, qi < N);
    }

    float m_run[kSub], l_run[kSub];
#pragma unroll
    for (int s = 0; s < kSub; ++s) { m_run[s] = -INFINITY; l_run[s] = 0.f; }

    const int last_key = min(N, (rt + 1) * kRowsPerBlock);      // exclusive
    const int n_tiles = (last_key + kStageRows - 1) / kStageRows;
    const float c = a.scale_log2e;

    StageRegs<T, D> pre;
    stage_load<T, D>(pre, K, 0, N);
    stage_store<T, D>(lds[0], pre);
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        if (t + 1 < n_tiles) stage_load<T, D>(pre, K, (t + 1) * kStageRows, N);
        const char* cur = lds[t & 1];
#pragma unroll
        for (int ks = 0; ks < kStageRows / 32; ++ks) {
            const int key0 = t * kStageRows + ks * 32;
            // wave-uniform: does any of this wave's queries see any of these keys?
            if (key0 > q0 + 32 * kSub - 1) continue;
            frag_t ak[kFrags];
#pragma unroll
            for (int f = 0; f < kFrags; ++f)
                ak[f] = *reinterpret_cast<const frag_t*>(cur + (ks * 32 + col) * kStride + f * 32 + half * 16);
#pragma unroll
            for (int s = 0; s < kSub; ++s) {
                const int qs0 = q0 + s * 32;
                if (key0 > qs0 + 31) continue;                   // wave-uniform
                f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < kFrags; ++f) mma<T>(acc, ak[f], bq[s][f]);
                const int qi = qs0 + col;
                if (key0 + 31 > qs0) {                           // tile crosses the diagonal
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (key0 + acc_row(r, half) > qi) acc[r] = -INFINITY;
                }
                float tmax = acc[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
                const float m_new = fmaxf(m_run[s], tmax * c);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += exp2_fast(__builtin_fmaf(acc[r], c, -m_use));
                l_run[s] = l_run[s] * exp2_fast(m_run[s] - m_use) + sum;
                m_run[s] = m_new;
            }
        }
        if (t + 1 < n_tiles) stage_store<T, D>(lds[(t + 1) & 1], pre);
        __syncthreads();
    }

    float* lse2 = a.lse2 + (size_t)(b * a.q_heads + h) * N;
    float* lse_nat = a.lse_opt ? a.lse_opt + (size_t)(b * a.q_heads + h) * N : nullptr;
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const float m_o = __shfl_xor(m_run[s], 32);
        const float l_o = __shfl_xor(l_run[s], 32);
        const float M = fmaxf(m_run[s], m_o);
        const float Mu = (M == -INFINITY) ? 0.f : M;
        const float L = l_run[s] * exp2_fast(m_run[s] - Mu) + l_o * exp2_fast(m_o - Mu);
        const float v = Mu + log2_fast(L);
        const int qi = q0 + s * 32 + col;
        if (half == 0 && qi < N) {
            lse2[qi] = v;
            if (lse_nat) lse_nat[qi] = v * 0.693147180559945309f;
        }
    }
}

// ------------------------------------------------------------------------------------
// Pass 2.  Block = (b, kv-head, tile of 4 * 32 * kSub keys, chunk of query rows).  Each
// wave keeps its keys in registers as the MFMA B operand (keys -> lanes) and streams the
// query rows of every q-head of the group through LDS as the A operand (rows ->
// accumulator registers), so a key's column sum is a per-lane scalar.  Row chunks bound
// the work per block (causal load balance) and let blocks that run together read the same
// Q rows; their partial sums are added in a fixed order by score_reduce_kernel.
// ------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void score_pass2_kernel(ScoreArgs a)
{
    constexpr int kSub = Sub<T>::kSub;
    constexpr int kStageRows = Sub<T>::kStageRows;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kStride = Tile<T, D>::kLdsStride;
    constexpr int kKeysPerBlock = kWavesPerBlock * 32 * kSub;

    __shared__ __attribute__((aligned(16))) char lds[2][kStageRows * kStride];
    __shared__ __attribute__((aligned(16))) float lds_lse[2][kStageRows];

    const int N = a.seq_len, W = a.window;
    const int G = a.q_heads / a.kv_heads;
    const int n_key_tiles = (N + kKeysPerBlock - 1) / kKeysPerBlock;
    const int n_chunks = a.n_chunks, R = a.chunk_rows;

    int bid = blockIdx.x;
    const int J = bid % n_key_tiles; bid /= n_key_tiles;
    const int I = n_chunks - 1 - (bid % n_chunks); bid /= n_chunks;
    const int bkv = bid;
    const int key_base = J * kKeysPerBlock;
    // rows of this chunk that can see any key of this tile
    const int r_begin = max(I * R, (key_base / kStageRows) * kStageRows);
    const int r_end = min((I + 1) * R, N);
    if (r_begin >= r_end) return;                 // block-uniform: pair above the diagonal

    const int b = bkv / a.kv_heads, kvh = bkv % a.kv_heads;
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    const int k0 = key_base + wave * 32 * kSub;

    frag_t bk[kSub][kFrags];
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const int kj = k0 + s * 32 + col;
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            bk[s][f] = load_frag_or_zero(K, (size_t)kj * Tile<T, D>::kRowBytes + f * 32 + half * 16, kj < N);
    }

    float glo[kSub], loc[kSub];
#pragma unroll
    for (int s = 0; s < kSub; ++s) { glo[s] = 0.f; loc[s] = 0.f; }

    const int tiles_per_head = (r_end - r_begin + kStageRows - 1) / kStageRows;
    const int n_tiles = tiles_per_head * G;
    const float c = a.scale_log2e;
    const int win0 = N - W;

    auto q_of = [&](int t) {
        const int g = t / tiles_per_head;
        return reinterpret_cast<const T*>(a.q) + ((size_t)(b * a.q_heads + kvh * G + g) * N) * D;
    };
    // row log-sum-exp: base-2 from pass 1's workspace, or the caller's natural-log one
    const float* lse_src = a.lse_in_nat ? a.lse_in_nat : a.lse2;
    const float lse_mul = a.lse_in_nat ? 1.44269504088896340736f : 1.0f;
    auto lse_of = [&](int t) {
        const int g = t / tiles_per_head;
        return lse_src + (size_t)(b * a.q_heads + kvh * G + g) * N;
    };
    auto row0_of = [&](int t) { return r_begin + (t % tiles_per_head) * kStageRows; };

    StageRegs<T, D> pre;
    float pre_lse = INFINITY;
    stage_load<T, D>(pre, q_of(0), row0_of(0), N);
    if (threadIdx.x < kStageRows) {
        const int r = row0_of(0) + threadIdx.x;
        pre_lse = r < N ? lse_of(0)[r] * lse_mul : INFINITY;
        lds_lse[0][threadIdx.x] = pre_lse;
    }
    stage_store<T, D>(lds[0], pre);
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        if (t + 1 < n_tiles) {
            stage_load<T, D>(pre, q_of(t + 1), row0_of(t + 1), N);
            if (threadIdx.x < kStageRows) {
                const int r = row0_of(t + 1) + threadIdx.x;
                pre_lse = r < N ? lse_of(t + 1)[r] * lse_mul : INFINITY;
            }
        }
        const char* cur = lds[t & 1];
        const float* cur_lse = lds_lse[t & 1];
        const int row_tile0 = row0_of(t);
#pragma unroll
        for (int rs = 0; rs < kStageRows / 32; ++rs) {
            const int row0 = row_tile0 + rs * 32;
            if (row0 + 31 < k0 || row0 >= N) continue;           // wave-uniform
            frag_t aq[kFrags];
#pragma unroll
            for (int f = 0; f < kFrags; ++f)
                aq[f] = *reinterpret_cast<const frag_t*>(cur + (rs * 32 + col) * kStride + f * 32 + half * 16);
            float lse_r[16];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(cur_lse + rs * 32 + 8 * q4 + 4 * half);
                lse_r[4 * q4 + 0] = v[0]; lse_r[4 * q4 + 1] = v[1];
                lse_r[4 * q4 + 2] = v[2]; lse_r[4 * q4 + 3] = v[3];
            }
            const bool in_window = row0 + 31 >= win0;            // wave-uniform
#pragma unroll
            for (int s = 0; s < kSub; ++s) {
                const int ks0 = k0 + s * 32;
                if (row0 + 31 < ks0) continue;                   // wave-uniform
                f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < kFrags; ++f) mma<T>(acc, aq[f], bk[s][f]);
                float p[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) p[r] = exp2_fast(__builtin_fmaf(acc[r], c, -lse_r[r]));
                if (row0 < ks0 + 31) {                           // tile crosses the diagonal
                    const int kj = ks0 + col;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (row0 + acc_row(r, half) < kj) p[r] = 0.f;
                }
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += p[r];
                glo[s] += sum;
                if (in_window) {
                    float lsum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        lsum += (row0 + acc_row(r, half) >= win0) ? p[r] : 0.f;
                    loc[s] += lsum;
                }
            }
        }
        if (t + 1 < n_tiles) {
            stage_store<T, D>(lds[(t + 1) & 1], pre);
            if (threadIdx.x < kStageRows) lds_lse[(t + 1) & 1][threadIdx.x] = pre_lse;
        }
        __syncthreads();
    }

    // the two half-waves hold disjoint row subsets of the same keys
    const int loc_chunk0 = a.loc_chunk0;
    float* out_glo = a.n_chunks == 1 ? a.s_glo + (size_t)bkv * N
                                     : a.part_glo + ((size_t)bkv * n_chunks + I) * N;
    float* out_loc = nullptr;
    if (a.n_chunks == 1) out_loc = a.s_loc + (size_t)bkv * N;
    else if (I >= loc_chunk0)
        out_loc = a.part_loc + ((size_t)bkv * (n_chunks - loc_chunk0) + (I - loc_chunk0)) * N;
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const float gsum = glo[s] + __shfl_xor(glo[s], 32);
        const float lsum = loc[s] + __shfl_xor(loc[s], 32);
        const int kj = k0 + s * 32 + col;
        if (half == 0 && kj < N) {
            out_glo[kj] = gsum;
            if (out_loc) out_loc[kj] = lsum;
        }
    }
}

// Adds the row-chunk partial sums of pass 2 in ascending chunk order (fixed order, so the
// result does not depend on scheduling).
__global__ __launch_bounds__(256) void score_reduce_kernel(ScoreArgs a, int keys_per_block)
{
    const int N = a.seq_len;
    const int bkv = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    const int key_base = (j / keys_per_block) * keys_per_block;
    const int first = key_base / a.chunk_rows;       // first chunk whose rows reach this key tile
    float g = 0.f, l = 0.f;
    for (int I = first; I < a.n_chunks; ++I) {
        g += a.part_glo[((size_t)bkv * a.n_chunks + I) * N + j];
        if (I >= a.loc_chunk0)
            l += a.part_loc[((size_t)bkv * (a.n_chunks - a.loc_chunk0) + (I - a.loc_chunk0)) * N + j];
    }
    a.s_glo[(size_t)bkv * N + j] = g;
    a.s_loc[(size_t)bkv * N + j] = l;
}

template <typename T> static int keys_per_block() { return kWavesPerBlock * 32 * Sub<T>::kSub; }

int score_keys_per_block(int dtype_is_f32) { return dtype_is_f32 ? keys_per_block<float>() : keys_per_block<bf16_t>(); }

template <typename T, int D>
static hipError_t launch_pass1_t(const ScoreArgs& a, hipStream_t st)
{
    constexpr int kRows = kWavesPerBlock * 32 * Sub<T>::kSub;
    const int BKV = a.batch * a.kv_heads, G = a.q_heads / a.kv_heads;
    const int n_row_tiles = (a.seq_len + kRows - 1) / kRows;
    const unsigned grid1 = (unsigned)(BKV * G * n_row_tiles);
    hipLaunchKernelGGL((score_pass1_kernel<T, D>), dim3(grid1), dim3(kBlock), 0, st, a);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_pass2_t(const ScoreArgs& a, hipStream_t st)
{
    constexpr int kKeys = kWavesPerBlock * 32 * Sub<T>::kSub;
    const int BKV = a.batch * a.kv_heads;
    const int n_key_tiles = (a.seq_len + kKeys - 1) / kKeys;
    const unsigned grid2 = (unsigned)(BKV * a.n_chunks * n_key_tiles);
    hipLaunchKernelGGL((score_pass2_kernel<T, D>), dim3(grid2), dim3(kBlock), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.n_chunks > 1) {
        dim3 g((a.seq_len + 255) / 256, BKV);
        hipLaunchKernelGGL(score_reduce_kernel, g, dim3(256), 0, st, a, kKeys);
        e = hipGetLastError();
    }
    return e;
}

#define EMS_DISPATCH(fn, a, f32, st)                                         \
    do {                                                                     \
        if (f32) {                                                           \
            if ((a).head_dim == 64) return fn<float, 64>(a, st);             \
            return fn<float, 128>(a, st);                                    \
        }                                                                    \
        if ((a).head_dim == 64) return fn<bf16_t, 64>(a, st);                \
        return fn<bf16_t, 128>(a, st);                                       \
    } while (0)

hipError_t launch_score_pass1(const ScoreArgs& a, bool f32, hipStream_t st) { EMS_DISPATCH(launch_pass1_t, a, f32, st); }
hipError_t launch_score_pass2(const ScoreArgs& a, bool f32, hipStream_t st) { EMS_DISPATCH(launch_pass2_t, a, f32, st); }

}  // namespace ems
