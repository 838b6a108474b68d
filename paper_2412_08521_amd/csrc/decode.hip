// Decode-time update of the compressed cache (Sec. 3.3, decoding paragraph; App. A,
// "Evict-then-Merge Details").
//
// decode_init_kernel  builds the per-token table (position, cache row, key norm, s_Glo,
//                     s_Loc^past, s_Loc^cur) from what the prefill compression returned.
// decode_step_kernel  one generated token: one block per (batch, kv-head) runs the whole
//                     step (for large caches the two sweeps over the cache rows are their own
//                     launches over row slices, see kPart) -- attention row of the new query over the expanded run-time
//                     cache (one dot product per cache ROW, shared by the tokens that share
//                     the entry; coalesced row loads, v_dot2 partials added with DPP),
//                     score accumulation, window ring shift, least important centre, its
//                     most similar centre, merge-or-evict with the look-up-table remap, new
//                     centre, past/cur swap.  Phases are separated by block barriers that
//                     every thread reaches.
#include "ems_common.h"
#include "ems_kernels.h"
#include "ems_rows.h"

namespace ems {

// ---- wave and block reductions.  Inside a wave the combine runs on DPP lane permutations
// (xor 1, xor 2 inside quads, then the half-row and row mirrors), which have ALU latency;
// the four row results are then read through scalar registers, so the result is uniform.
// all 16 lanes of every row end up with their row's result
template <bool kMax>
__device__ __forceinline__ float row_reduce(float v)
{
    v = comb<kMax>(v, dpp_f<kDppXor1>(v));
    v = comb<kMax>(v, dpp_f<kDppXor2>(v));
    v = comb<kMax>(v, dpp_f<kDppHalfMirror>(v));
    v = comb<kMax>(v, dpp_f<kDppMirror>(v));
    return v;
}
template <bool kMax>
__device__ __forceinline__ float wave_reduce(float v)
{
    v = row_reduce<kMax>(v);
    return comb<kMax>(comb<kMax>(lane_value(v, 0), lane_value(v, 16)), comb<kMax>(lane_value(v, 32), lane_value(v, 48)));
}

// Every thread of the block must call; the result is identical in every thread.
template <int kWaves, int kN, bool kMax>
__device__ __forceinline__ void block_reduce(float (&v)[kN], float (*buf)[kWaves])
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int i = 0; i < kN; ++i) v[i] = wave_reduce<kMax>(v[i]);
    __syncthreads();                                    // buf free again
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < kN; ++i) buf[i][wave] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kN; ++i) {
        if constexpr (kWaves == 16) {
            v[i] = lane_value(row_reduce<kMax>(buf[i][lane & 15]), 0);
        } else {
            float r = buf[i][0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) r = comb<kMax>(r, buf[i][w]);       // fixed order
            v[i] = r;
        }
    }
}
// arg-min (kMin) or arg-max of (value, index) pairs, lowest index on ties; index < 0 = none
template <bool kMin>
__device__ __forceinline__ bool better(float v, int i, float bv, int bi)
{
    if (i < 0) return false;
    if (bi < 0) return true;
    if (kMin ? v < bv : v > bv) return true;
    return v == bv && i < bi;
}
template <bool kMin, int kCtrl>
__device__ __forceinline__ void arg_step(float& v, int& i)
{
    const float ov = dpp_f<kCtrl>(v);
    const int oi = dpp_i<kCtrl>(i);
    if (better<kMin>(ov, oi, v, i)) { v = ov; i = oi; }
}
template <bool kMin>
__device__ __forceinline__ void row_arg(float& v, int& i)
{
    arg_step<kMin, kDppXor1>(v, i);
    arg_step<kMin, kDppXor2>(v, i);
    arg_step<kMin, kDppHalfMirror>(v, i);
    arg_step<kMin, kDppMirror>(v, i);
}
template <int kWaves, bool kMin>
__device__ __forceinline__ void block_arg(float& v, int& i, float* fbuf, int* ibuf)
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    row_arg<kMin>(v, i);
    {
        float bv = lane_value(v, 0);
        int bi = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
        for (int r = 16; r < 64; r += 16) {
            const float ov = lane_value(v, r);
            const int oi = __builtin_amdgcn_readlane(i, r);
            if (better<kMin>(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        v = bv; i = bi;
    }
    __syncthreads();
    if (lane == 0) { fbuf[wave] = v; ibuf[wave] = i; }
    __syncthreads();
    if constexpr (kWaves == 16) {
        v = fbuf[lane & 15]; i = ibuf[lane & 15];
        row_arg<kMin>(v, i);
        v = lane_value(v, 0); i = __builtin_amdgcn_readlane(i, 0);
    } else {
        v = fbuf[0]; i = ibuf[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w)
            if (better<kMin>(fbuf[w], ibuf[w], v, i)) { v = fbuf[w]; i = ibuf[w]; }
    }
}

// dot product of the 8 bf16 elements of two 16-byte row pieces, f32 accumulation
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot8_bf16(const frag_t& x, const frag_t& y)
{
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, x), b = __builtin_bit_cast(bf16x8_t, y);
    float acc = 0.f;
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), acc, false);
    return acc;
}

// register `idx` (0..15) of a 32x32 accumulator, idx not known at compile time
__device__ __forceinline__ float acc_pick(const f32x16_t& acc, int idx)
{
    float v = acc[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) v = idx == r ? acc[r] : v;
    return v;
}

// ------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_init_kernel(DecodeInitArgs a)
{
    const int n_imp = a.n_imp, E = a.n_imp + a.n_tbm, W = a.window, Nb = a.budget, N = a.seq_len;
    const int Tn = E + W;
    const int bkv = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= Tn) return;

    int pos = -1, row = -1;
    float norm = 0.f;
    if (j < n_imp) {
        pos = a.kept_pos[(size_t)bkv * Nb + j];
        row = j;
        norm = a.k_norm[(size_t)bkv * E + j];
        a.st.row_norm[(size_t)bkv * Nb + j] = norm;
        a.st.entry_tok[(size_t)bkv * n_imp + j] = j;
        a.st.entry_count[(size_t)bkv * n_imp + j] = a.slot_count[(size_t)bkv * (n_imp + 1) + j];
    } else if (j < E) {
        const int i = j - n_imp;
        const int d = a.tbm_dest[(size_t)bkv * a.n_tbm + i];
        if (d >= 0 && d < n_imp) {
            pos = a.tbm_idx[(size_t)bkv * a.n_tbm + i];
            row = d;
            norm = a.k_norm[(size_t)bkv * E + j];
        }
    } else {
        row = n_imp + (j - E);
        pos = a.kept_pos[(size_t)bkv * Nb + row];
        const T* kr = reinterpret_cast<const T*>(a.st.k_cache) + ((size_t)bkv * (Nb + 1) + row) * D;
        float ss = 0.f;
        for (int d = 0; d < D; ++d) { const float x = to_float(kr[d]); ss = __builtin_fmaf(x, x, ss); }
        norm = sqrtf(ss);
        a.st.row_norm[(size_t)bkv * Nb + row] = norm;
    }
    const size_t o = (size_t)bkv * Tn + j;
    const bool live = row >= 0;
    const int cp = min(max(pos, 0), N - 1);
    a.st.tok_pos[o] = live ? pos : -1;
    a.st.tok_row[o] = row;
    a.st.tok_norm[o] = norm;
    a.st.tok_glo[o] = live ? a.s_glo[(size_t)bkv * N + cp] : 0.f;
    a.st.tok_past[o] = live ? a.s_loc[(size_t)bkv * N + cp] : 0.f;
    a.st.tok_cur[o] = 0.f;
    if (bkv == 0 && j == 0) *a.st.step_count = 0;
}

// ------------------------------------------------------------------------------------
// kPart = 0: one block per (batch, kv-head) runs the whole step, kBlock = 256 (the step is a chain
// of short dependent phases, and every instruction a wave spends on a block-wide bookkeeping
// step is paid once per wave).
// Large caches: one compute unit cannot pull the cache rows fast enough, so the step is four
// launches in stream order, the two row sweeps cut into slices of a.slice_rows rows:
//   kPart = 1  phase 1 (row dots)           grid (slices, heads), 256 threads
//   kPart = 2  phases 2-4                    grid (1, heads), 1024 threads
//   kPart = 3  phase 5 (centre cosines)      grid (slices, heads), 256 threads
//   kPart = 4  phases 6-7                    grid (1, heads), 1024 threads
// (Letting the last cosine block of a head run phases 6-7 itself saves a launch and was measured
// slower: the next launch's latency hides behind the sweep anyway.)
// What one part leaves for the next lives in the workspace: the staged dots and row norms, and a
// small hand-over record per head (kHand* offsets below).
// Dynamic LDS (floats): dot[G][budget] | rn[budget] when that fits, else the same arrays
// live in the caller's workspace (a.lds_floats == 0).
constexpr int kHandSelf = 0;       // [8]  new query . new key per q-head (log2 units)
constexpr int kHandNewNorm = 8;    //      norm of the new key
constexpr int kHandOldSc = 9;      // [4]  scalars of the token that left the window
constexpr int kHandOldPos = 13;    //      its position (int)
constexpr int kHandStar = 14;      //      the least important centre (int)
constexpr int kHandStep = 15;      //      tokens generated before this one (int)
constexpr int kHandPart = 16;      // [kDecodeMaxSlices][2] best cosine and its centre per slice
constexpr int kHandOldRow = kHandPart + 2 * kDecodeMaxSlices;   // key row, then value row, of that token

template <typename T, int D, int G, int kBlock, int kPart>
__global__ __launch_bounds__(kBlock) void decode_step_kernel(DecodeStepArgs a)
{
    constexpr bool kAll = kPart == 0;
    constexpr bool kDoDots = kAll || kPart == 1, kDoSoftmax = kAll || kPart == 2;
    constexpr bool kDoCos = kAll || kPart == 3;
    static_assert(kPart >= 0 && kPart <= 4, "parts");
    static_assert(kHandOldRow % 4 == 0 && kHandOldRow + 2 * D * (int)sizeof(T) / 4 <= kDecodeHandFloats, "hand-over record");
    using P = Pack<T>;
    constexpr int kE = P::kElems;
    constexpr int kWaves = kBlock / kWave;
    constexpr int kLpr = Tile<T, D>::kChunksPerRow;          // lanes per cache row
    constexpr int kFrags = Tile<T, D>::kFrags;               // MFMA operand fragments per row
    constexpr int kRowBytes = Tile<T, D>::kRowBytes;
    constexpr int kUnroll = 4;                               // independent loads in flight per thread
    constexpr int kPre = kBlock == 256 ? 2 : 1;              // row tiles in flight per wave
    constexpr bool kPreload = (kAll && kBlock == 256) || kPart == 2;   // first batch of table elements fetched up front

    extern __shared__ float dyn_lds[];
    __shared__ float fbuf[kWaves];
    __shared__ int ibuf[kWaves];
    __shared__ float vbuf[G < 2 ? 2 : G][kWaves];            // vector reductions
    __shared__ float sq[kWaves][32];                         // squared norms of a wave's row tile
    __shared__ float sh_self[G];                             // new query . new key (log2 units)
    __shared__ frag_t old_k[kLpr], old_v[kLpr];              // the token that leaves the window
    __shared__ float old_sc[4];                              // its norm, glo, past, cur
    __shared__ int old_pos;
    __shared__ float sh_newnorm;

    const int n_imp = a.n_imp, E = a.n_imp + a.n_tbm, W = a.window, Nb = a.budget;
    const int Tn = E + W;
    const int bkv = blockIdx.y, slice = blockIdx.x;          // slice = 0 unless the part sweeps rows
    const int tid = threadIdx.x;
    // tokens generated before this one: the caller's count, or the counter kept in the state.  The
    // counter is advanced after every block has read it: by a separate launch after the one-launch
    // step; in the sliced step the first part copies it into every head's hand-over record,
    // the later parts read that copy, and the last part advances it.
    const int step = a.step >= 0 ? a.step
                   : (kPart >= 2 ? reinterpret_cast<const int*>(a.hand + (size_t)bkv * kDecodeHandFloats)[kHandStep] : *a.st.step_count);
    const int lane = tid % kWave, wave = tid / kWave;
    const int col = lane & 31, half = lane >> 5;             // MFMA operand row / k-half of this lane
    const int grp = tid / kLpr, piece = tid % kLpr;

    char* Kc = reinterpret_cast<char*>(a.st.k_cache) + (size_t)bkv * (Nb + 1) * D * sizeof(T);
    char* Vc = reinterpret_cast<char*>(a.st.v_cache) + (size_t)bkv * (Nb + 1) * D * sizeof(T);
    float* row_norm = a.st.row_norm + (size_t)bkv * Nb;
    int32_t* entry_count = a.st.entry_count + (size_t)bkv * n_imp;
    int32_t* entry_tok = a.st.entry_tok + (size_t)bkv * n_imp;
    int32_t* tok_pos = a.st.tok_pos + (size_t)bkv * Tn;
    int32_t* tok_row = a.st.tok_row + (size_t)bkv * Tn;
    float* tok_norm = a.st.tok_norm + (size_t)bkv * Tn;
    float* tok_glo = a.st.tok_glo + (size_t)bkv * Tn;
    float* tok_past = a.st.tok_past + (size_t)bkv * Tn;
    float* tok_cur = a.st.tok_cur + (size_t)bkv * Tn;
    // the sweeping parts write the staged arrays to the workspace; the part that consumes them
    // copies them into LDS first when they fit
    float* ws_stage = a.ws + (size_t)bkv * ((size_t)(G + 1) * Nb);
    const bool in_lds = a.lds_floats > 0 && (kAll || kPart == 2);   // block-uniform
    float* stage = in_lds ? dyn_lds : ws_stage;
    float* hand = kAll ? nullptr : a.hand + (size_t)bkv * kDecodeHandFloats;
    int* hand_i = reinterpret_cast<int*>(hand);
    frag_t* hand_row = reinterpret_cast<frag_t*>(hand + kHandOldRow);
    // rows of this block's sweeps: every row, or the block's slice
    const int r_lo = kAll ? 0 : slice * a.slice_rows;
    const int r_end = kAll ? Nb + 1 : min(r_lo + a.slice_rows, Nb + 1);       // phase 1 (row Nb = the new key)
    const int c_end = kAll ? n_imp : min(r_lo + a.slice_rows, n_imp);        // phase 5
    float* dot = stage;                                      // [G][budget] q_g . cache row
    float* rn_of = stage + (size_t)G * Nb;                   // [budget] copy of row_norm
    const char* qn = reinterpret_cast<const char*>(a.q_new) + (size_t)bkv * G * D * sizeof(T);
    const char* kn = reinterpret_cast<const char*>(a.k_new) + (size_t)bkv * D * sizeof(T);
    const char* vn = reinterpret_cast<const char*>(a.v_new) + (size_t)bkv * D * sizeof(T);

    // ---- phase 1: q_g . (every cache row), the new token's own key included as row Nb ----
    // bf16: a row is kLpr consecutive lanes x 16 bytes, so a wave-wide load covers 64 / kLpr
    // whole rows (fully coalesced); each lane forms the partial dots of its 8 elements with
    // v_dot2 and the kLpr partials are added with DPP.  One dot per cache ROW serves every
    // token that shares the entry.
    // f32 (validation mode): MFMA contraction, 32 cache rows per tile as the A operand, the
    // group's q-heads in B columns 0..G-1.
    // Everything this thread will need from global memory that does not depend on earlier
    // phases is requested here, behind the first row loads, so that the round trips overlap:
    // the first batch of table elements (all of them for small tables), the centre token of
    // "its" entry, its share of the row norms, the new token's row.
    constexpr bool kDot2 = sizeof(T) == 2;
    constexpr int kRowsPerWave = kWave / kLpr;               // whole rows per wave-wide load
    constexpr int kRowsPerPass = kWaves * kRowsPerWave;
    constexpr int kInFlight = kBlock == 1024 ? 8 : 4;        // row loads in flight per lane (bf16 path)
    const int sub = lane / kLpr;                             // this lane's row within the wave's load
    constexpr int kCt = kBlock == 1024 ? 2 : 1;              // centre tokens looked up ahead per thread (phase 4)
    int ct_pre[kCt];
#pragma unroll
    for (int u = 0; u < kCt; ++u) ct_pre[u] = (kDoSoftmax && tid + u * kBlock < n_imp) ? entry_tok[tid + u * kBlock] : 0;
    frag_t new_k = zero_frag(), new_v = zero_frag();
    float m[G], sum[G];
    float tot2[2] = {0.f, 0.f};                              // sum of s_Glo, sum of s_Loc
    float self_tot = 0.f;
    int s_star = 0, f = 0;
    float cv = 0.f;
    int ci = -1;
    int pre_rr[kUnroll];
    float pre_tn[kUnroll], pre_tg[kUnroll], pre_tp[kUnroll], pre_tc[kUnroll];
    auto preload_table = [&]() {
#pragma unroll
        for (int u = 0; u < (kPreload ? kUnroll : 0); ++u) {
            const int j = tid + u * kBlock;
            const bool ok = j < Tn;
            pre_rr[u] = ok ? tok_row[j] : -1;
            pre_tn[u] = ok ? tok_norm[j] : 0.f;
            pre_tg[u] = ok ? tok_glo[j] : 0.f;
            pre_tp[u] = ok ? tok_past[j] : 0.f;
            pre_tc[u] = ok ? tok_cur[j] : 0.f;
        }
    };
    if constexpr (kDoDots) {
    if constexpr (kDot2) {
        frag_t qp[G];
#pragma unroll
        for (int g = 0; g < G; ++g) qp[g] = *reinterpret_cast<const frag_t*>(qn + ((size_t)g * kLpr + piece) * 16);
        new_k = *reinterpret_cast<const frag_t*>(kn + piece * 16);
        frag_t fk[kInFlight];
        auto load_rows = [&](int r0) {
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int r = r0 + u * kRowsPerPass;
                fk[u] = r < Nb ? *reinterpret_cast<const frag_t*>(Kc + ((size_t)r * kLpr + piece) * 16) : new_k;
            }
        };
        const int r_first = r_lo + wave * kRowsPerWave + sub;
        load_rows(r_first);
        preload_table();
        const float rn_mine = (kAll && tid < Nb) ? row_norm[tid] : 0.f;
        if (grp == 0) new_v = *reinterpret_cast<const frag_t*>(vn + piece * 16);
        for (int r0 = r_first; r0 < r_end; r0 += kRowsPerPass * kInFlight) {
            if (r0 != r_first) load_rows(r0);
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int r = r0 + u * kRowsPerPass;
                if (r >= r_end) break;                       // uniform over the row's lanes
                float d[G];
#pragma unroll
                for (int g = 0; g < G; ++g) d[g] = group_sum<kLpr>(dot8_bf16(fk[u], qp[g]));
                if (piece == 0) {
                    if (r < Nb) {
#pragma unroll
                        for (int g = 0; g < G; ++g) dot[(size_t)g * Nb + r] = d[g];
                    } else {
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            sh_self[g] = a.scale_log2e * d[g];
                            if (!kAll) hand[kHandSelf + g] = a.scale_log2e * d[g];
                        }
                    }
                }
            }
        }
        for (int r = r_lo + tid; r < min(r_end, Nb); r += kBlock) rn_of[r] = (kAll && r == tid) ? rn_mine : row_norm[r];
        if (grp == 0 && (kAll || slice == 0)) {
            const float ss = group_sum<kLpr>(frag_sumsq<T>(new_k));
            if (piece == 0) { sh_newnorm = sqrtf(ss); if (!kAll) hand[kHandNewNorm] = sqrtf(ss); }
        }
    } else {
        frag_t bq[kFrags];
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            bq[f] = load_frag_or_zero(qn, (size_t)col * kRowBytes + f * 32 + half * 16, col < G);
        const int t_lo = r_lo / 32, n_tiles = (r_end + 31) / 32;      // slices are whole tiles
        frag_t fa[kPre][kFrags];
        auto load_tiles = [&](int t0) {
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                const int r = (t0 + u * kWaves) * 32 + col;
                const char* src = r < Nb ? Kc + (size_t)r * kRowBytes : kn;
#pragma unroll
                for (int f = 0; f < kFrags; ++f) fa[u][f] = load_frag_or_zero(src, f * 32 + half * 16, r <= Nb);
            }
        };
        load_tiles(t_lo + wave);
        preload_table();
        const float rn_mine = (kAll && tid < Nb) ? row_norm[tid] : 0.f;
        if (grp == 0) {
            new_k = *reinterpret_cast<const frag_t*>(kn + piece * 16);
            new_v = *reinterpret_cast<const frag_t*>(vn + piece * 16);
        }
        for (int t0 = t_lo + wave; t0 < n_tiles; t0 += kWaves * kPre) {
            if (t0 != t_lo + wave) load_tiles(t0);
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                const int t = t0 + u * kWaves;
                if (t >= n_tiles) break;                     // wave-uniform
                f32x16_t acc;
                mma_first<T>(acc, fa[u][0], bq[0]);
#pragma unroll
                for (int f = 1; f < kFrags; ++f) mma<T>(acc, fa[u][f], bq[f]);
                if (col < G) {
#pragma unroll
                    for (int r16 = 0; r16 < 16; ++r16) {
                        const int row = t * 32 + acc_row(r16, half);
                        if (row < Nb) dot[(size_t)col * Nb + row] = acc[r16];
                        else if (row == Nb) {
                            sh_self[col] = a.scale_log2e * acc[r16];
                            if (!kAll) hand[kHandSelf + col] = a.scale_log2e * acc[r16];
                        }
                    }
                }
            }
        }
        for (int r = r_lo + tid; r < min(r_end, Nb); r += kBlock) rn_of[r] = (kAll && r == tid) ? rn_mine : row_norm[r];
        if (grp == 0 && (kAll || slice == 0)) {
            const float ss = group_sum<kLpr>(frag_sumsq<T>(new_k));
            if (piece == 0) { sh_newnorm = sqrtf(ss); if (!kAll) hand[kHandNewNorm] = sqrtf(ss); }
        }
    }
    }   // kDoDots
    if constexpr (kPart == 1) {
        if (slice == 0 && tid == 0) hand_i[kHandStep] = step;
        return;
    }
    if constexpr (kPart == 2) {
        // what the dots launch left: the new token's own logits and norm, the staged arrays
        preload_table();
        if (tid < G) sh_self[tid] = hand[kHandSelf + tid];
        if (tid == 0) sh_newnorm = hand[kHandNewNorm];
        if (grp == 0) {
            new_k = *reinterpret_cast<const frag_t*>(kn + piece * 16);
            new_v = *reinterpret_cast<const frag_t*>(vn + piece * 16);
        }
        if (in_lds) {
            constexpr int kCopy = 8;                         // loads in flight per thread
            for (int i0 = tid; i0 < (G + 1) * Nb; i0 += kBlock * kCopy) {
                float t[kCopy];
#pragma unroll
                for (int u = 0; u < kCopy; ++u) t[u] = i0 + u * kBlock < (G + 1) * Nb ? ws_stage[i0 + u * kBlock] : 0.f;
#pragma unroll
                for (int u = 0; u < kCopy; ++u)
                    if (i0 + u * kBlock < (G + 1) * Nb) dyn_lds[i0 + u * kBlock] = t[u];
            }
        }
    }
    if constexpr (kDoSoftmax) {
    __syncthreads();

    // ---- phase 2: softmax over the live tokens and the new token (Eq. 1) ---------------
    // logit of token j in row r: scale * (|k_j| / |centre of r|) * (q . row r).  Three light
    // sweeps over the table: maxima, sums, weights.
#pragma unroll
    for (int g = 0; g < G; ++g) m[g] = sh_self[g];
    for (int j0 = tid; j0 < Tn; j0 += kBlock * kUnroll) {
        int rr[kUnroll];
        float tn[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            if (kPreload && j0 == tid) { rr[u] = pre_rr[u]; tn[u] = pre_tn[u]; }
            else { rr[u] = j < Tn ? tok_row[j] : -1; tn[u] = j < Tn ? tok_norm[j] : 0.f; }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = rr[u];
            if (r < 0) continue;
            const float rn = rn_of[r];
            const float c = a.scale_log2e * (rn > 0.f ? tn[u] / rn : 0.f);
#pragma unroll
            for (int g = 0; g < G; ++g) m[g] = fmaxf(m[g], c * dot[(size_t)g * Nb + r]);
        }
    }
    block_reduce<kWaves, G, true>(m, vbuf);
#pragma unroll
    for (int g = 0; g < G; ++g) sum[g] = tid == 0 ? exp2_fast(sh_self[g] - m[g]) : 0.f;
    for (int j0 = tid; j0 < Tn; j0 += kBlock * kUnroll) {
        int rr[kUnroll];
        float tn[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            if (kPreload && j0 == tid) { rr[u] = pre_rr[u]; tn[u] = pre_tn[u]; }
            else { rr[u] = j < Tn ? tok_row[j] : -1; tn[u] = j < Tn ? tok_norm[j] : 0.f; }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = rr[u];
            if (r < 0) continue;
            const float rn = rn_of[r];
            const float c = a.scale_log2e * (rn > 0.f ? tn[u] / rn : 0.f);
#pragma unroll
            for (int g = 0; g < G; ++g) sum[g] += exp2_fast(c * dot[(size_t)g * Nb + r] - m[g]);
        }
    }
    block_reduce<kWaves, G, false>(sum, vbuf);
#pragma unroll
    for (int g = 0; g < G; ++g) sum[g] = 1.0f / sum[g];
    // accumulate the row into s_Glo and s_Loc^cur (Sec. 3.3); the sums that Eq. 2 needs
    // (phase 4) are those of the updated scalars
    for (int j0 = tid; j0 < Tn; j0 += kBlock * kUnroll) {
        int rr[kUnroll];
        float tn[kUnroll], tg[kUnroll], tp[kUnroll], tc[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            const bool ok = j < Tn;
            if (kPreload && j0 == tid) { rr[u] = pre_rr[u]; tn[u] = pre_tn[u]; tg[u] = pre_tg[u]; tp[u] = pre_tp[u]; tc[u] = pre_tc[u]; }
            else {
                rr[u] = ok ? tok_row[j] : -1;
                tn[u] = ok ? tok_norm[j] : 0.f;
                tg[u] = ok ? tok_glo[j] : 0.f;
                tp[u] = ok ? tok_past[j] : 0.f;
                tc[u] = ok ? tok_cur[j] : 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            if (j >= Tn) break;
            const int r = rr[u];
            float w[G];
            if (r >= 0) {
                const float rn = rn_of[r];
                const float c = a.scale_log2e * (rn > 0.f ? tn[u] / rn : 0.f);
                float tot = 0.f;
#pragma unroll
                for (int g = 0; g < G; ++g) { w[g] = exp2_fast(c * dot[(size_t)g * Nb + r] - m[g]) * sum[g]; tot += w[g]; }
                const float glo = tg[u] + tot, cur = tc[u] + tot;
                tok_glo[j] = glo;
                tok_cur[j] = cur;
                tot2[0] += glo;
                tot2[1] += tp[u] + cur;
            } else {
#pragma unroll
                for (int g = 0; g < G; ++g) w[g] = 0.f;
            }
            if (a.attn_opt) {
#pragma unroll
                for (int g = 0; g < G; ++g) a.attn_opt[((size_t)bkv * G + g) * (Tn + 1) + j] = w[g];
            }
        }
    }
#pragma unroll                                               // self_tot: every thread, same value
    for (int g = 0; g < G; ++g) {
        const float w = exp2_fast(sh_self[g] - m[g]) * sum[g];
        self_tot += w;
        if (a.attn_opt && tid == 0) a.attn_opt[((size_t)bkv * G + g) * (Tn + 1) + Tn] = w;
    }
    if (tid == 0) { tot2[0] += self_tot; tot2[1] += self_tot; }   // the new token: glo = cur = its own weight
    block_reduce<kWaves, 2, false>(tot2, vbuf);              // also: every token's scalars are written

    // ---- phase 3: the oldest window token leaves, the new token takes its ring slot ----
    const int ring = step % W;
    const int jo = E + ring, ro = n_imp + ring;
    if (grp == 0) {
        old_k[piece] = *reinterpret_cast<const frag_t*>(Kc + ((size_t)ro * kLpr + piece) * 16);
        old_v[piece] = *reinterpret_cast<const frag_t*>(Vc + ((size_t)ro * kLpr + piece) * 16);
        *reinterpret_cast<frag_t*>(Kc + ((size_t)ro * kLpr + piece) * 16) = new_k;
        *reinterpret_cast<frag_t*>(Vc + ((size_t)ro * kLpr + piece) * 16) = new_v;
    }
    if (tid == 0) {
        old_pos = tok_pos[jo];
        old_sc[0] = tok_norm[jo]; old_sc[1] = tok_glo[jo]; old_sc[2] = tok_past[jo]; old_sc[3] = tok_cur[jo];
        tok_pos[jo] = a.seq_len + step; tok_row[jo] = ro; tok_norm[jo] = sh_newnorm;
        tok_glo[jo] = self_tot; tok_past[jo] = 0.f; tok_cur[jo] = self_tot;
        row_norm[ro] = sh_newnorm;
    }

    // ---- phase 4: least important class centre (Eq. 2 on the tokens' scalars) ----------
    const float align = tot2[0] > 0.f ? tot2[1] / tot2[0] : 0.f;
    float bv = 0.f;
    int bi = -1;
    for (int s0 = tid; s0 < n_imp; s0 += kBlock * kCt) {
        float cg[kCt], cp[kCt], cc[kCt];
#pragma unroll
        for (int u = 0; u < kCt; ++u) {                      // every gather requested before the first is used
            const int s = s0 + u * kBlock;
            const int ct = s0 == tid ? ct_pre[u] : (s < n_imp ? entry_tok[s] : 0);
            cg[u] = tok_glo[ct]; cp[u] = tok_past[ct]; cc[u] = tok_cur[ct];
        }
#pragma unroll
        for (int u = 0; u < kCt; ++u) {
            const int s = s0 + u * kBlock;
            const float sc = fmaxf(cg[u] * align, cp[u] + cc[u]);
            if (s < n_imp && better<true>(sc, s, bv, bi)) { bv = sc; bi = s; }
        }
    }
    block_arg<kWaves, true>(bv, bi, fbuf, ibuf);             // its barriers also publish phase 3
    s_star = max(bi, 0);                                     // block-uniform, in [0, n_imp)
    }   // kDoSoftmax
    if constexpr (kPart == 2) {
        if (grp == 0) { hand_row[piece] = old_k[piece]; hand_row[kLpr + piece] = old_v[piece]; }
        if (tid == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hand[kHandOldSc + i] = old_sc[i];
            hand_i[kHandOldPos] = old_pos;
            hand_i[kHandStar] = s_star;
        }
        return;
    }
    if constexpr (kPart >= 3) s_star = hand_i[kHandStar];
    f = entry_tok[s_star];

    // ---- phase 5: its most similar other centre (Eq. 5, cosine of the stored keys) -----
    // bf16: per entry row the dot with the chosen row and the row's own squared norm, again as
    // v_dot2 partials added with DPP.  f32: two MFMA chains per tile of 32 entries -- tile x
    // (chosen row in every column) for the dots, tile x tile for the squared norms on its
    // diagonal.
    if constexpr (kDoCos) {
    if constexpr (kDot2) {
        const frag_t sp = *reinterpret_cast<const frag_t*>(Kc + ((size_t)s_star * kLpr + piece) * 16);
        const float rn_star = inv_norm(group_sum<kLpr>(dot8_bf16(sp, sp)));
        const int s_first = r_lo + wave * kRowsPerWave + sub;
        for (int s0 = s_first; s0 < c_end; s0 += kRowsPerPass * kInFlight) {
            frag_t fk[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int s = s0 + u * kRowsPerPass;
                fk[u] = load_frag_or_zero(Kc, ((size_t)s * kLpr + piece) * 16, s < c_end);
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int s = s0 + u * kRowsPerPass;
                if (s >= c_end) break;                       // uniform over the row's lanes
                const float d = group_sum<kLpr>(dot8_bf16(fk[u], sp));
                const float e2 = group_sum<kLpr>(dot8_bf16(fk[u], fk[u]));
                const float sim = (d * inv_norm(e2)) * rn_star;
                if (piece == 0 && s != s_star && better<false>(sim, s, cv, ci)) { cv = sim; ci = s; }
            }
        }
    } else
    {
        frag_t bs[kFrags];
        float ss = 0.f;
#pragma unroll
        for (int fr = 0; fr < kFrags; ++fr) {
            bs[fr] = *reinterpret_cast<const frag_t*>(Kc + (size_t)s_star * kRowBytes + fr * 32 + half * 16);
            ss += frag_sumsq<T>(bs[fr]);
        }
        ss += __shfl_xor(ss, 32);
        const float rn_star = inv_norm(ss);
        const int t_lo = r_lo / 32, n_tiles = (c_end + 31) / 32;
        const int pick = col & 15;                           // the accumulator register this lane judges
        const int my_local = acc_row(pick, half);            // ... and the tile row it belongs to
        const bool diag_here = half == ((col >> 2) & 1);     // this lane holds |row col|^2 ...
        const int diag_reg = 4 * (col >> 3) + (col & 3);     // ... in this register
        for (int t0 = t_lo + wave; t0 < n_tiles; t0 += kWaves * kPre) {
            frag_t fa[kPre][kFrags];
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                const int r = (t0 + u * kWaves) * 32 + col;
#pragma unroll
                for (int fr = 0; fr < kFrags; ++fr)
                    fa[u][fr] = load_frag_or_zero(Kc, (size_t)r * kRowBytes + fr * 32 + half * 16, r < c_end);
            }
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                const int t = t0 + u * kWaves;
                if (t >= n_tiles) break;                     // wave-uniform
                f32x16_t acc, acc2;
                mma_first<T>(acc, fa[u][0], bs[0]);
                mma_first<T>(acc2, fa[u][0], fa[u][0]);
#pragma unroll
                for (int fr = 1; fr < kFrags; ++fr) { mma<T>(acc, fa[u][fr], bs[fr]); mma<T>(acc2, fa[u][fr], fa[u][fr]); }
                __builtin_amdgcn_wave_barrier();             // the previous tile's sq[] has been read
                if (diag_here) sq[wave][col] = acc_pick(acc2, diag_reg);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int s = t * 32 + my_local;
                const float sim = (acc_pick(acc, pick) * inv_norm(sq[wave][my_local])) * rn_star;
                if (col < 16 && s < c_end && s != s_star && better<false>(sim, s, cv, ci)) { cv = sim; ci = s; }
            }
        }
    }
    }   // kDoCos
    if constexpr (kPart == 4) {
        // the slices' winners (combined below, lowest centre on ties) and the token that left the window
        cv = tid < a.n_slices ? hand[kHandPart + 2 * tid] : 0.f;
        ci = tid < a.n_slices ? hand_i[kHandPart + 2 * tid + 1] : -1;
        if (grp == 0) { old_k[piece] = hand_row[piece]; old_v[piece] = hand_row[kLpr + piece]; }
        if (tid == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) old_sc[i] = hand[kHandOldSc + i];
            old_pos = hand_i[kHandOldPos];
        }
    }
    block_arg<kWaves, false>(cv, ci, fbuf, ibuf);
    if constexpr (kPart == 3) {
        if (tid == 0) { hand[kHandPart + 2 * slice] = cv; hand_i[kHandPart + 2 * slice + 1] = ci; }
        return;
    }
    const bool merged = ci >= 0 && cv > a.tau;
    const int dst = merged ? ci : -1;

    // ---- phase 6: merge at class-centre level, or evict; followers follow --------------
    if (merged && grp == 0) {
        const float ca = (float)entry_count[s_star], cb = (float)entry_count[dst];
        const float na = row_norm[s_star], nb = row_norm[dst];
        const float ra = na > 0.f ? 1.0f / na : 0.f, rb = nb > 0.f ? 1.0f / nb : 0.f;
        float ka[kE], kb[kE], va[kE], vb[kE];
        P::unpack(*reinterpret_cast<const frag_t*>(Kc + ((size_t)s_star * kLpr + piece) * 16), ka);
        P::unpack(*reinterpret_cast<const frag_t*>(Kc + ((size_t)dst * kLpr + piece) * 16), kb);
        P::unpack(*reinterpret_cast<const frag_t*>(Vc + ((size_t)s_star * kLpr + piece) * 16), va);
        P::unpack(*reinterpret_cast<const frag_t*>(Vc + ((size_t)dst * kLpr + piece) * 16), vb);
#pragma unroll
        for (int i = 0; i < kE; ++i) {
            kb[i] = nb * ((cb * (kb[i] * rb) + ca * (ka[i] * ra)) / (ca + cb));
            vb[i] = (cb * vb[i] + ca * va[i]) / (ca + cb);
        }
        *reinterpret_cast<frag_t*>(Kc + ((size_t)dst * kLpr + piece) * 16) = P::pack(kb);
        *reinterpret_cast<frag_t*>(Vc + ((size_t)dst * kLpr + piece) * 16) = P::pack(vb);
    }
    for (int j0 = tid; j0 < E; j0 += kBlock * kUnroll) {
        int rr[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            rr[u] = j < E ? tok_row[j] : -1;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int j = j0 + u * kBlock;
            if (rr[u] != s_star || j == f) continue;
            if (merged) {
                tok_row[j] = dst;
            } else {
                tok_row[j] = -1; tok_pos[j] = -1;
                tok_norm[j] = 0.f; tok_glo[j] = 0.f; tok_past[j] = 0.f; tok_cur[j] = 0.f;
            }
        }
    }
    __syncthreads();                                         // entry s_star fully read
    // the token that left the window is the new centre of entry s_star and takes the
    // departed centre's table element
    if (grp == 0) {
        *reinterpret_cast<frag_t*>(Kc + ((size_t)s_star * kLpr + piece) * 16) = old_k[piece];
        *reinterpret_cast<frag_t*>(Vc + ((size_t)s_star * kLpr + piece) * 16) = old_v[piece];
    }
    if (tid == 0) {
        if (merged) entry_count[dst] += entry_count[s_star];
        entry_count[s_star] = 1;
        row_norm[s_star] = old_sc[0];
        tok_pos[f] = old_pos; tok_row[f] = s_star; tok_norm[f] = old_sc[0];
        tok_glo[f] = old_sc[1]; tok_past[f] = old_sc[2]; tok_cur[f] = old_sc[3];
        if (a.decision_opt) { a.decision_opt[(size_t)bkv * 2] = s_star; a.decision_opt[(size_t)bkv * 2 + 1] = dst; }
        if (a.sim_opt) a.sim_opt[bkv] = ci >= 0 ? cv : -INFINITY;
    }
    __syncthreads();

    // ---- phase 7: a full window of queries: s_Loc^cur becomes s_Loc^past (Sec. 3.3) ----
    if ((step + 1) % W == 0) {
        for (int j = tid; j < Tn; j += kBlock) { tok_past[j] = tok_cur[j]; tok_cur[j] = 0.f; }
    }
    if constexpr (kPart == 4) {
        if (bkv == 0 && tid == 0) *a.st.step_count = step + 1;   // every block of the step reads the hand-over copy
    }
}

__global__ void decode_bump_kernel(int32_t* step_count, int step)
{
    *step_count = (step >= 0 ? step : *step_count) + 1;
}

// ------------------------------------------------------------------------------------
template <typename T, int D>
static hipError_t launch_decode_init_t(const DecodeInitArgs& a, hipStream_t st)
{
    const int Tn = a.n_imp + a.n_tbm + a.window;
    hipLaunchKernelGGL((decode_init_kernel<T, D>), dim3((Tn + 255) / 256, a.bkv), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_decode_init(const DecodeInitArgs& a, bool f32, hipStream_t st)
{
    if (f32) return a.head_dim == 64 ? launch_decode_init_t<float, 64>(a, st) : launch_decode_init_t<float, 128>(a, st);
    return a.head_dim == 64 ? launch_decode_init_t<bf16_t, 64>(a, st) : launch_decode_init_t<bf16_t, 128>(a, st);
}

template <typename T, int D, int kBlock, int kPart>
static hipError_t launch_decode_part(const DecodeStepArgs& a, hipStream_t st)
{
    const bool sweeps = kPart == 1 || kPart == 3;
    const dim3 g(sweeps ? a.n_slices : 1, a.bkv), b(kBlock);
    const size_t lds = (kPart == 0 || kPart == 2) ? sizeof(float) * (size_t)a.lds_floats : 0;
    switch (a.group) {
        case 1: hipLaunchKernelGGL((decode_step_kernel<T, D, 1, kBlock, kPart>), g, b, lds, st, a); break;
        case 2: hipLaunchKernelGGL((decode_step_kernel<T, D, 2, kBlock, kPart>), g, b, lds, st, a); break;
        case 4: hipLaunchKernelGGL((decode_step_kernel<T, D, 4, kBlock, kPart>), g, b, lds, st, a); break;
        case 8: hipLaunchKernelGGL((decode_step_kernel<T, D, 8, kBlock, kPart>), g, b, lds, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Whether the step runs as four launches over row slices, and how the rows are cut.  f32 rows
// need twice the operand registers: the validation mode always takes the one-block kernel.
bool decode_split(int budget, int n_imp, int n_tbm, int window, bool f32, int* slice_rows, int* n_slices)
{
    *slice_rows = 0; *n_slices = 1;
    if (f32 || (budget <= 512 && n_imp + n_tbm + window <= 2048)) return false;
    const int tiles = (budget + 1 + 31) / 32;                     // 32-row tiles, the new key's row included
    int per = 4;                                                  // 128 rows per slice ...
    while ((tiles + per - 1) / per > kDecodeMaxSlices) per *= 2;  // ... unless that makes too many slices
    *slice_rows = per * 32;
    *n_slices = (tiles + per - 1) / per;
    return true;
}

template <typename T, int D>
static hipError_t launch_decode_step_t(const DecodeStepArgs& a, hipStream_t st)
{
    hipError_t e;
    if (a.n_slices > 1 || a.slice_rows > 0) {
        if constexpr (sizeof(T) == 2) {
            e = launch_decode_part<T, D, 256, 1>(a, st);
            if (e == hipSuccess) e = launch_decode_part<T, D, 1024, 2>(a, st);
            if (e == hipSuccess) e = launch_decode_part<T, D, 256, 3>(a, st);
            if (e == hipSuccess) e = launch_decode_part<T, D, 1024, 4>(a, st);
        } else {
            return hipErrorInvalidValue;
        }
    } else {
        e = launch_decode_part<T, D, 256, 0>(a, st);
    }
    if (e != hipSuccess || a.slice_rows > 0) return e;           // the sliced step advances the counter itself
    hipLaunchKernelGGL(decode_bump_kernel, dim3(1), dim3(1), 0, st, a.st.step_count, a.step);
    return hipGetLastError();
}

hipError_t launch_decode_step(const DecodeStepArgs& a, bool f32, hipStream_t st)
{
    if (f32) return a.head_dim == 64 ? launch_decode_step_t<float, 64>(a, st) : launch_decode_step_t<float, 128>(a, st);
    return a.head_dim == 64 ? launch_decode_step_t<bf16_t, 64>(a, st) : launch_decode_step_t<bf16_t, 128>(a, st);
}

}  // namespace ems
