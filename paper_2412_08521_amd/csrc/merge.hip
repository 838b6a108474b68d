// Head-wise evict-then-merge (Sec. 4.2, Eq. 5, App. A).
//
// dest_kernel     for every to-be-merged (TBM) token: cosine similarity of its key with
//                 the class-centre keys as an MFMA contraction of the raw keys, scaled by
//                 the reciprocal norms afterwards, with the row arg-max fused into the
//                 accumulator read-out; similarity not above tau -> zero class.  With many
//                 centres the centre list is cut into slices, one block per (128 tokens,
//                 slice), and dest_combine_kernel takes the best slice per token.
// merge_kernel    one wave per output row: a centre slot gathers the TBM tokens sent to it
//                 in ascending order and averages (unit keys scaled by the centre's norm,
//                 raw values); one block per head does the same for the zero class; the
//                 local-window rows are copied.  Every output element has exactly one
//                 writer, so there are no atomics and results are reproducible bit for bit.
#include "ems_common.h"
#include "ems_kernels.h"
#include "ems_rows.h"

namespace ems {

constexpr int kMrgWaves = 4;
constexpr int kMrgBlock = kMrgWaves * kWave;
constexpr int kDestDepth = 4;        // centre stages whose rows a block has in flight at once
constexpr int kDestMaxSlices = 16;   // centre slices per head at most
constexpr int kMergeWaves = 8;       // output rows per merge block
constexpr int kMergeBlock = kMergeWaves * kWave;
constexpr int kMergePiece = 4096;    // TBM tokens whose destinations a merge block holds in LDS

template <typename T> struct DestCfg { static constexpr int kStageRows = 64; };
template <> struct DestCfg<float> { static constexpr int kStageRows = 32; };

__device__ __forceinline__ int clamp_pos(int p, int n) { return min(max(p, 0), n - 1); }

// ------------------------------------------------------------------------------------
// Destination of every TBM token (Eq. 5, then the threshold).  The redundancy is the key
// cosine, the value cosine or their product (Sec. 4.1; similarity ablation of App. B):
// kSim = 0 / 1 / 2, i.e. one or two sources, each with its own MFMA contraction.
// Block = (128 TBM tokens, one (b, kv-head)); each wave keeps 32 TBM rows in registers as
// the MFMA B operand (tokens -> lanes) and the centre rows stream through LDS as the A
// operand (centres -> accumulator registers), so the running arg-max is a per-lane pair.
// ------------------------------------------------------------------------------------
template <typename T, int D, int kSim>
__global__ __launch_bounds__(kMrgBlock) void dest_kernel(MergeArgs a)
{
    constexpr int kStageRows = DestCfg<T>::kStageRows;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kStride = Tile<T, D>::kLdsStride;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kPerThread = kCpr * kStageRows / kMrgBlock;
    constexpr int kSrc = kSim == 2 ? 2 : 1;

    __shared__ __attribute__((aligned(16))) char lds[kSrc][kStageRows * kStride];
    __shared__ __attribute__((aligned(16))) float lds_rn[kSrc][kStageRows];

    const int N = a.seq_len, n_imp = a.n_imp, n_tbm = a.n_tbm;
    const int bkv = blockIdx.z, slice = blockIdx.y;
    const int c_begin = slice * a.slice_rows, c_end = min(n_imp, c_begin + a.slice_rows);   // this block's centres
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;
    const T* V = reinterpret_cast<const T*>(a.v) + ((size_t)bkv * N) * D;
    const T* src[kSrc];
    if constexpr (kSim == 0) { src[0] = K; }
    else if constexpr (kSim == 1) { src[0] = V; }
    else { src[0] = K; src[1] = V; }
    const int32_t* imp = a.imp_idx + (size_t)bkv * n_imp;
    const int32_t* tbm = a.tbm_idx + (size_t)bkv * n_tbm;

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    const int ti = blockIdx.x * (kMrgWaves * 32) + wave * 32 + col;   // this lane's TBM token
    const bool t_ok = ti < n_tbm;
    const int t_pos = t_ok ? clamp_pos(tbm[ti], N) : 0;

    frag_t bt[kSrc][kFrags];
    float t_rn[kSrc];
    float k_sumsq = 0.f;
#pragma unroll
    for (int s = 0; s < kSrc; ++s) {
        float ss = 0.f;
#pragma unroll
        for (int f = 0; f < kFrags; ++f) {
            bt[s][f] = load_frag_or_zero(src[s], (size_t)t_pos * Tile<T, D>::kRowBytes + f * 32 + half * 16, t_ok);
            ss += frag_sumsq<T>(bt[s][f]);
        }
        ss += __shfl_xor(ss, 32);
        t_rn[s] = inv_norm(ss);
        if (kSim != 1 && s == 0) k_sumsq = ss;
    }
    if constexpr (kSim == 1) {                                      // the key norm is an output in every mode
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            k_sumsq += frag_sumsq<T>(load_frag_or_zero(K, (size_t)t_pos * Tile<T, D>::kRowBytes + f * 32 + half * 16, t_ok));
        k_sumsq += __shfl_xor(k_sumsq, 32);
    }

    float best = -INFINITY;
    int arg = 0;

    // A round is kDestDepth stages of kStageRows centres.  All of a round's centre positions,
    // then all of its rows, are requested before the first stage is used: two global round
    // trips per round, however many stages it has.
    for (int r0 = c_begin; r0 < c_end; r0 += kDestDepth * kStageRows) {
        int pos_pf[kDestDepth][kPerThread];
        frag_t pf[kDestDepth][kSrc][kPerThread];
#pragma unroll
        for (int st = 0; st < kDestDepth; ++st)
#pragma unroll
            for (int i = 0; i < kPerThread; ++i) {
                const int ci = r0 + st * kStageRows + (threadIdx.x + i * kMrgBlock) / kCpr;
                pos_pf[st][i] = ci < c_end ? clamp_pos(imp[ci], N) : -1;
            }
#pragma unroll
        for (int st = 0; st < kDestDepth; ++st)
#pragma unroll
            for (int i = 0; i < kPerThread; ++i) {
                const int cc = (threadIdx.x + i * kMrgBlock) % kCpr;
#pragma unroll
                for (int s = 0; s < kSrc; ++s)
                    pf[st][s][i] = load_frag_or_zero(src[s], ((size_t)max(pos_pf[st][i], 0) * kCpr + cc) * 16, pos_pf[st][i] >= 0);
            }
#pragma unroll
        for (int st = 0; st < kDestDepth; ++st) {
            const int c0 = r0 + st * kStageRows;
            if (c0 >= c_end) break;                            // block-uniform
            __syncthreads();                                   // previous tile fully consumed
#pragma unroll
            for (int i = 0; i < kPerThread; ++i) {
                const int c = threadIdx.x + i * kMrgBlock;
                const int row = c / kCpr, cc = c % kCpr;
#pragma unroll
                for (int s = 0; s < kSrc; ++s) {
                    *reinterpret_cast<frag_t*>(lds[s] + row * kStride + cc * 16) = pf[st][s][i];
                    // the kCpr consecutive lanes that hold one row add up its squares
                    const float ss = group_sum<kCpr>(frag_sumsq<T>(pf[st][s][i]));
                    if (cc == 0) lds_rn[s][row] = inv_norm(ss);
                }
            }
            __syncthreads();
#pragma unroll
            for (int rs = 0; rs < kStageRows / 32; ++rs) {
                const int cbase = c0 + rs * 32;
                if (cbase >= c_end) continue;                  // block-uniform
                f32x16_t acc[kSrc];
#pragma unroll
                for (int s = 0; s < kSrc; ++s) {
                    acc[s] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int f = 0; f < kFrags; ++f) {
                        const frag_t ac = *reinterpret_cast<const frag_t*>(lds[s] + (rs * 32 + col) * kStride + f * 32 + half * 16);
                        mma<T>(acc[s], ac, bt[s][f]);
                    }
                }
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4_t rn[kSrc];
#pragma unroll
                    for (int s = 0; s < kSrc; ++s)
                        rn[s] = *reinterpret_cast<const f32x4_t*>(lds_rn[s] + rs * 32 + 8 * q4 + 4 * half);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int ci = cbase + 8 * q4 + 4 * half + e;
                        float sim = (acc[0][4 * q4 + e] * rn[0][e]) * t_rn[0];
                        if constexpr (kSrc == 2) sim *= (acc[1][4 * q4 + e] * rn[1][e]) * t_rn[1];
                        if (ci < c_end && sim > best) { best = sim; arg = ci; }
                    }
                }
            }
        }
    }
    // the other half-wave looked at the other centres of every tile
    const float best_o = __shfl_xor(best, 32);
    const int arg_o = __shfl_xor(arg, 32);
    if (best_o > best || (best_o == best && arg_o < arg)) { best = best_o; arg = arg_o; }
    if (half == 0 && t_ok) {
        if (a.n_slices == 1) {
            a.tbm_sim[(size_t)bkv * n_tbm + ti] = best;
            a.tbm_dest[(size_t)bkv * n_tbm + ti] = best > a.tau ? arg : a.budget;
        } else {
            a.part_best[((size_t)bkv * a.n_slices + slice) * n_tbm + ti] = best;
            a.part_arg[((size_t)bkv * a.n_slices + slice) * n_tbm + ti] = arg;
        }
        if (slice == 0) a.k_norm[(size_t)bkv * (n_imp + n_tbm) + n_imp + ti] = sqrtf(k_sumsq);
    }
}

// The best slice of every TBM token (lowest slice, hence lowest centre, on ties), then the
// threshold.  One thread per token.
__global__ __launch_bounds__(kMrgBlock) void dest_combine_kernel(MergeArgs a)
{
    const int bkv = blockIdx.y, ti = blockIdx.x * kMrgBlock + threadIdx.x;
    if (ti >= a.n_tbm) return;
    const float* pb = a.part_best + (size_t)bkv * a.n_slices * a.n_tbm + ti;
    const int32_t* pa = a.part_arg + (size_t)bkv * a.n_slices * a.n_tbm + ti;
    float b[kDestMaxSlices];
    int g[kDestMaxSlices];
#pragma unroll
    for (int s = 0; s < kDestMaxSlices; ++s) {               // every slice requested before the first compare
        const bool on = s < a.n_slices;
        b[s] = on ? pb[(size_t)s * a.n_tbm] : -INFINITY;
        g[s] = on ? pa[(size_t)s * a.n_tbm] : 0;
    }
    float best = -INFINITY;
    int arg = 0;
#pragma unroll
    for (int s = 0; s < kDestMaxSlices; ++s)
        if (b[s] > best) { best = b[s]; arg = g[s]; }
    a.tbm_sim[(size_t)bkv * a.n_tbm + ti] = best;
    a.tbm_dest[(size_t)bkv * a.n_tbm + ti] = best > a.tau ? arg : a.budget;
}

// ------------------------------------------------------------------------------------
// Segmented average.  A row of D elements is 16-byte pieces over kLpr lanes, so one wave
// has kGroups = 64 / kLpr rows in flight per load; members of a slot are dealt to the
// groups in ascending order and the groups are added by a fixed butterfly at the end.
// ------------------------------------------------------------------------------------
template <typename T, int D>
struct RowAcc {
    static constexpr int kE = Pack<T>::kElems;
    static constexpr int kLpr = Tile<T, D>::kChunksPerRow;     // lanes per row
    static constexpr int kGroups = kWave / kLpr;
    float k[kE], v[kE];
    float wsum;                                                // weighted merge only
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < kE; ++i) { k[i] = 0.f; v[i] = 0.f; }
        wsum = 0.f;
    }
    static __device__ __forceinline__ frag_t load_piece(const T* X, int pos, int piece)
    {
        return *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(X) + ((size_t)pos * kLpr + piece) * 16);
    }
    // adds a token given its key and value pieces (unit key, raw value); returns the key's
    // norm.  All kLpr lanes of the group must call together.
    __device__ __forceinline__ float accumulate(const frag_t& fk, const frag_t& fv)
    {
        const float ss = group_sum<kLpr>(frag_sumsq<T>(fk));
        const float rn = inv_norm(ss);
        float xk[kE], xv[kE];
        Pack<T>::unpack(fk, xk);
        Pack<T>::unpack(fv, xv);
#pragma unroll
        for (int i = 0; i < kE; ++i) { k[i] = __builtin_fmaf(xk[i], rn, k[i]); v[i] += xv[i]; }
        return sqrtf(ss);
    }
    // the same with weight w >= 0 on the token (score-weighted merge, Sec. 4.2)
    __device__ __forceinline__ float accumulate_weighted(const frag_t& fk, const frag_t& fv, float w)
    {
        const float ss = group_sum<kLpr>(frag_sumsq<T>(fk));
        const float rnw = inv_norm(ss) * w;
        float xk[kE], xv[kE];
        Pack<T>::unpack(fk, xk);
        Pack<T>::unpack(fv, xv);
#pragma unroll
        for (int i = 0; i < kE; ++i) { k[i] = __builtin_fmaf(xk[i], rnw, k[i]); v[i] = __builtin_fmaf(xv[i], w, v[i]); }
        wsum += w;
        return sqrtf(ss);
    }
    __device__ __forceinline__ float add(const T* K, const T* V, int pos, int piece)
    {
        return accumulate(load_piece(K, pos, piece), load_piece(V, pos, piece));
    }
    __device__ __forceinline__ float add_weighted(const T* K, const T* V, int pos, int piece, float w)
    {
        return accumulate_weighted(load_piece(K, pos, piece), load_piece(V, pos, piece), w);
    }
    // adds the groups together: afterwards every group holds the total
    template <bool kWeighted>
    __device__ __forceinline__ void reduce_groups()
    {
#pragma unroll
        for (int o = kLpr; o < kWave; o <<= 1) {
#pragma unroll
            for (int i = 0; i < kE; ++i) { k[i] += __shfl_xor(k[i], o); v[i] += __shfl_xor(v[i], o); }
            if constexpr (kWeighted) wsum += __shfl_xor(wsum, o);
        }
    }
};

// Walks the staged TBM tokens (`len` of them: destination and position in LDS) in chunks
// `first, first+step, ...` of 64, adds those whose destination is `target` to `acc` and
// returns how many there were.
template <typename T, int D, bool kWeighted>
__device__ __forceinline__ int gather_members(RowAcc<T, D>& acc, const T* K, const T* V, const float* Wt,
                                              const int* ldest, const int* lpos, int len, int target,
                                              int first, int step, int* wlist)
{
    constexpr int kLpr = RowAcc<T, D>::kLpr, kGroups = RowAcc<T, D>::kGroups;
    const int lane = threadIdx.x % kWave;
    const int grp = lane / kLpr, piece = lane % kLpr;
    const int n_chunks = (len + kWave - 1) / kWave;
    int count = 0;
    for (int ch = first; ch < n_chunks; ch += step) {
        const int i = ch * kWave + lane;
        const bool match = i < len && ldest[i] == target;
        const unsigned long long mask = __ballot(match);
        if (mask == 0ull) continue;                              // wave-uniform
        const int n = __popcll(mask);
        if (match) wlist[__popcll(mask & ((1ull << lane) - 1ull))] = lpos[i];
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        // kInFlight members per lane group at a time, all their loads issued before the first is
        // added; a group still adds its members in ascending order
        constexpr int kInFlight = 4;
        for (int m0 = 0; m0 < n; m0 += kGroups * kInFlight) {
            frag_t fk[kInFlight], fv[kInFlight];
            float w[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int m = m0 + u * kGroups + grp;
                const int pos = m < n ? wlist[m] : 0;
                fk[u] = load_frag_or_zero(K, ((size_t)pos * kLpr + piece) * 16, m < n);
                fv[u] = load_frag_or_zero(V, ((size_t)pos * kLpr + piece) * 16, m < n);
                w[u] = (kWeighted && m < n) ? fmaxf(Wt[pos], 0.f) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                if (m0 + u * kGroups + grp >= n) break;
                if constexpr (kWeighted) acc.accumulate_weighted(fk[u], fv[u], w[u]);
                else acc.accumulate(fk[u], fv[u]);
            }
        }
        __builtin_amdgcn_wave_barrier();
        count += n;
    }
    return count;
}

template <typename T, int D, bool kWeighted>
__global__ __launch_bounds__(kMergeBlock) void merge_kernel(MergeArgs a)
{
    using Acc = RowAcc<T, D>;
    constexpr int kE = Acc::kE, kLpr = Acc::kLpr;

    // destinations and positions of a piece of the TBM list, shared by the block's rows
    __shared__ int ldest[kMergePiece];
    __shared__ int lpos[kMergePiece];
    __shared__ int wlist_all[kMergeWaves][kWave];
    __shared__ float zsum[kMergeWaves][2][D];
    __shared__ int zcnt[kMergeWaves];
    __shared__ float zwsum[kMergeWaves];

    const int N = a.seq_len, W = a.window, Nb = a.budget, n_imp = a.n_imp, n_tbm = a.n_tbm;
    const int bkv = blockIdx.y;
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;
    const T* V = reinterpret_cast<const T*>(a.v) + ((size_t)bkv * N) * D;
    T* Ko = reinterpret_cast<T*>(a.k_out) + ((size_t)bkv * (Nb + 1)) * D;
    T* Vo = reinterpret_cast<T*>(a.v_out) + ((size_t)bkv * (Nb + 1)) * D;
    const int32_t* imp = a.imp_idx + (size_t)bkv * n_imp;
    const int32_t* tbm = n_tbm ? a.tbm_idx + (size_t)bkv * n_tbm : nullptr;
    const int32_t* dest = n_tbm ? a.tbm_dest + (size_t)bkv * n_tbm : nullptr;
    int32_t* kept = a.kept_pos + (size_t)bkv * Nb;
    int32_t* cnt = a.slot_count + (size_t)bkv * (n_imp + 1);
    const float* Wt = kWeighted ? a.weight + (size_t)bkv * N : nullptr;

    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int grp = lane / kLpr, piece = lane % kLpr;
    int* wlist = wlist_all[wave];

    // what this wave produces: block 0 is the zero class (its waves split the TBM list), every
    // other wave owns one output row: a class-centre slot, a local-window row, or nothing
    const bool zero_class = blockIdx.x == 0;
    const int job = zero_class ? -1 : (blockIdx.x - 1) * kMergeWaves + wave;     // wave-uniform
    const bool centre = !zero_class && job < n_imp;
    const bool local = !zero_class && job >= n_imp && job < n_imp + W;

    if (local) {
        // ---- local-window row: copied unchanged
        const int pos = N - W + (job - n_imp);
        if (grp == 0) {
            const frag_t fk = *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(K) + ((size_t)pos * kLpr + piece) * 16);
            const frag_t fv = *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(V) + ((size_t)pos * kLpr + piece) * 16);
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Ko) + ((size_t)job * kLpr + piece) * 16) = fk;
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Vo) + ((size_t)job * kLpr + piece) * 16) = fv;
        }
        if (lane == 0) kept[job] = pos;
    }

    // ---- class-centre slot: the centre itself is the first member
    Acc acc; acc.clear();
    int c_pos = 0;
    float c_norm = 0.f;
    frag_t raw_k = zero_frag(), raw_v = zero_frag();
    if (centre) {
        c_pos = clamp_pos(imp[job], N);
        if (grp == 0) {
            raw_k = *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(K) + ((size_t)c_pos * kLpr + piece) * 16);
            raw_v = *reinterpret_cast<const frag_t*>(reinterpret_cast<const char*>(V) + ((size_t)c_pos * kLpr + piece) * 16);
            if constexpr (kWeighted) c_norm = acc.accumulate_weighted(raw_k, raw_v, fmaxf(Wt[c_pos], 0.f));
            else c_norm = acc.accumulate(raw_k, raw_v);
        }
        c_norm = __shfl(c_norm, 0);
    }

    // ---- the TBM list goes through LDS a piece at a time; every wave takes its members from it
    int joined = 0;
    for (int p0 = 0; p0 < n_tbm; p0 += kMergePiece) {
        const int len = min(kMergePiece, n_tbm - p0);
        if (p0 > 0) __syncthreads();                       // the previous piece is consumed
        for (int i = threadIdx.x; i < len; i += kMergeBlock) {
            ldest[i] = dest[p0 + i];
            lpos[i] = clamp_pos(tbm[p0 + i], N);
        }
        __syncthreads();
        if (centre) joined += gather_members<T, D, kWeighted>(acc, K, V, Wt, ldest, lpos, len, job, 0, 1, wlist);
        else if (zero_class) joined += gather_members<T, D, kWeighted>(acc, K, V, Wt, ldest, lpos, len, Nb, wave, kMergeWaves, wlist);
    }

    if (centre) {
        const int members = 1 + joined;
        acc.template reduce_groups<kWeighted>();
        if (grp == 0) {
            frag_t out_k = raw_k, out_v = raw_v;                      // nobody joined: exact copy
            const float m = kWeighted ? acc.wsum : (float)members;    // total weight of the entry
            if (members > 1 && m > 0.f) {
                float ok[kE], ov[kE];
#pragma unroll
                for (int i = 0; i < kE; ++i) { ok[i] = c_norm * (acc.k[i] / m); ov[i] = acc.v[i] / m; }
                out_k = Pack<T>::pack(ok);
                out_v = Pack<T>::pack(ov);
            }
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Ko) + ((size_t)job * kLpr + piece) * 16) = out_k;
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Vo) + ((size_t)job * kLpr + piece) * 16) = out_v;
        }
        if (lane == 0) {
            kept[job] = c_pos;
            cnt[job] = members;
            a.k_norm[(size_t)bkv * (n_imp + n_tbm) + job] = c_norm;
        }
    }

    if (zero_class) {
        // ---- zero class: every wave has added its share in order; wave 0 adds the waves in order
        acc.template reduce_groups<kWeighted>();
        if (grp == 0) {
#pragma unroll
            for (int i = 0; i < kE; ++i) { zsum[wave][0][piece * kE + i] = acc.k[i]; zsum[wave][1][piece * kE + i] = acc.v[i]; }
        }
        if (lane == 0) { zcnt[wave] = joined; zwsum[wave] = acc.wsum; }
        __syncthreads();
        if (wave == 0 && grp == 0) {
            int total = 0;
            float wtot = 0.f;
            for (int w = 0; w < kMergeWaves; ++w) { total += zcnt[w]; wtot += zwsum[w]; }
            const float denom = kWeighted ? wtot : (float)total;     // members, or their total weight
            float ok[kE], ov[kE];
#pragma unroll
            for (int i = 0; i < kE; ++i) {
                float sk = 0.f, sv = 0.f;
                for (int w = 0; w < kMergeWaves; ++w) { sk += zsum[w][0][piece * kE + i]; sv += zsum[w][1][piece * kE + i]; }
                ok[i] = denom > 0.f ? sk / denom : 0.f;
                ov[i] = denom > 0.f ? sv / denom : 0.f;
            }
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Ko) + ((size_t)Nb * kLpr + piece) * 16) = Pack<T>::pack(ok);
            *reinterpret_cast<frag_t*>(reinterpret_cast<char*>(Vo) + ((size_t)Nb * kLpr + piece) * 16) = Pack<T>::pack(ov);
            if (lane == 0) cnt[n_imp] = total;
        }
    }
}

// ------------------------------------------------------------------------------------
// Shared-entry expansion (App. A): one 16-lane group per output row; a merged token's key
// is its entry's key rescaled from the centre's norm to the token's own norm.
// ------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kMrgBlock) void expand_kernel(ExpandArgs a)
{
    using Acc = RowAcc<T, D>;
    constexpr int kE = Acc::kE, kLpr = Acc::kLpr, kGroups = Acc::kGroups;
    const int n_imp = a.n_imp, n_tbm = a.n_tbm, Nb = a.budget;
    const int n_exp = n_imp + n_tbm + a.window;
    const int bkv = blockIdx.y;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int grp = lane / kLpr, piece = lane % kLpr;
    const int row = (blockIdx.x * kMrgWaves + wave) * kGroups + grp;
    if (row >= n_exp) return;

    const char* Kc = reinterpret_cast<const char*>(a.k_cache) + (size_t)bkv * (Nb + 1) * D * sizeof(T);
    const char* Vc = reinterpret_cast<const char*>(a.v_cache) + (size_t)bkv * (Nb + 1) * D * sizeof(T);
    char* Ke = reinterpret_cast<char*>(a.k_exp) + ((size_t)bkv * n_exp + row) * D * sizeof(T);
    char* Ve = reinterpret_cast<char*>(a.v_exp) + ((size_t)bkv * n_exp + row) * D * sizeof(T);

    int src = -1, pos = -1;          // cache row the token lives in
    float scale = 1.f;
    bool rescale = false;
    if (row < n_imp) {
        src = row; pos = a.kept_pos[(size_t)bkv * Nb + row];
    } else if (row < n_imp + n_tbm) {
        const int i = row - n_imp;
        const int s = a.tbm_dest[(size_t)bkv * n_tbm + i];
        if (s >= 0 && s < n_imp) {
            const float nc = a.k_norm[(size_t)bkv * (n_imp + n_tbm) + s];
            const float ni = a.k_norm[(size_t)bkv * (n_imp + n_tbm) + n_imp + i];
            src = s; pos = a.tbm_idx[(size_t)bkv * n_tbm + i];
            scale = nc > 0.f ? ni / nc : 0.f;
            rescale = true;
        }
    } else {
        src = n_imp + (row - n_imp - n_tbm); pos = a.kept_pos[(size_t)bkv * Nb + src];
    }
    frag_t fk = zero_frag(), fv = zero_frag();
    if (src >= 0) {
        fk = *reinterpret_cast<const frag_t*>(Kc + ((size_t)src * kLpr + piece) * 16);
        fv = *reinterpret_cast<const frag_t*>(Vc + ((size_t)src * kLpr + piece) * 16);
        if (rescale) {
            float x[kE];
            Pack<T>::unpack(fk, x);
#pragma unroll
            for (int e = 0; e < kE; ++e) x[e] *= scale;
            fk = Pack<T>::pack(x);
        }
    }
    *reinterpret_cast<frag_t*>(Ke + piece * 16) = fk;
    *reinterpret_cast<frag_t*>(Ve + piece * 16) = fv;
    if (piece == 0) a.pos_exp[(size_t)bkv * n_exp + row] = pos;
}

template <typename T, int D>
static hipError_t launch_expand_t(const ExpandArgs& a, hipStream_t st)
{
    const int rows_per_block = kMrgWaves * RowAcc<T, D>::kGroups;
    const int n_exp = a.n_imp + a.n_tbm + a.window;
    dim3 g((n_exp + rows_per_block - 1) / rows_per_block, a.bkv);
    hipLaunchKernelGGL((expand_kernel<T, D>), g, dim3(kMrgBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_expand(const ExpandArgs& a, bool f32, hipStream_t st)
{
    if (f32) {
        if (a.head_dim == 64) return launch_expand_t<float, 64>(a, st);
        return launch_expand_t<float, 128>(a, st);
    }
    if (a.head_dim == 64) return launch_expand_t<bf16_t, 64>(a, st);
    return launch_expand_t<bf16_t, 128>(a, st);
}

// How the centre list is cut for dest_kernel: rows per slice (whole rounds) and slices.
void dest_slicing(int n_imp, bool f32, int* slice_rows, int* n_slices)
{
    const int round_rows = kDestDepth * (f32 ? DestCfg<float>::kStageRows : DestCfg<bf16_t>::kStageRows);
    const int rounds = (max(n_imp, 1) + round_rows - 1) / round_rows;
    const int per_slice = (rounds + kDestMaxSlices - 1) / kDestMaxSlices;
    *slice_rows = per_slice * round_rows;
    *n_slices = (rounds + per_slice - 1) / per_slice;
}

template <typename T, int D>
static hipError_t launch_evict_merge_t(const MergeArgs& a, hipStream_t st)
{
    hipError_t e = hipSuccess;
    if (a.n_tbm > 0) {
        dim3 g((a.n_tbm + kMrgWaves * 32 - 1) / (kMrgWaves * 32), a.n_slices, a.bkv);
        if (a.similarity == 0) hipLaunchKernelGGL((dest_kernel<T, D, 0>), g, dim3(kMrgBlock), 0, st, a);
        else if (a.similarity == 1) hipLaunchKernelGGL((dest_kernel<T, D, 1>), g, dim3(kMrgBlock), 0, st, a);
        else hipLaunchKernelGGL((dest_kernel<T, D, 2>), g, dim3(kMrgBlock), 0, st, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (a.n_slices > 1) {
            dim3 gc((a.n_tbm + kMrgBlock - 1) / kMrgBlock, a.bkv);
            hipLaunchKernelGGL(dest_combine_kernel, gc, dim3(kMrgBlock), 0, st, a);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    const int jobs = a.n_imp + a.window;
    dim3 g(1 + (jobs + kMergeWaves - 1) / kMergeWaves, a.bkv);
    if (a.weight) hipLaunchKernelGGL((merge_kernel<T, D, true>), g, dim3(kMergeBlock), 0, st, a);
    else hipLaunchKernelGGL((merge_kernel<T, D, false>), g, dim3(kMergeBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_evict_merge(const MergeArgs& a, bool f32, hipStream_t st)
{
    if (f32) {
        if (a.head_dim == 64) return launch_evict_merge_t<float, 64>(a, st);
        return launch_evict_merge_t<float, 128>(a, st);
    }
    if (a.head_dim == 64) return launch_evict_merge_t<bf16_t, 64>(a, st);
    return launch_evict_merge_t<bf16_t, 128>(a, st);
}

}  // namespace ems
