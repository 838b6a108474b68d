// Decode-time update of the compressed cache (Sec. 3.2, decoding paragraph; App. A,
// "Evict-then-Merge Details").
//
// decode_init_kernel  builds the per-token table (position, cache row, key norm, s_Glo,
//                     s_Loc^past, s_Loc^cur) from what the prefill compression returned.
// decode_step_kernel  one generated token: one 1024-thread block per (batch, kv-head) runs
//                     the whole step -- attention row of the new query over the expanded
//                     run-time cache (one dot product per cache ROW, shared by the tokens
//                     that share the entry), score accumulation, window ring shift, least
//                     important centre, its most similar centre, merge-or-evict with the
//                     look-up-table remap, new centre, past/cur swap.  Phases are separated
//                     by block barriers that every thread reaches.
#include "ems_common.h"
#include "ems_kernels.h"
#include "ems_rows.h"

namespace ems {

constexpr int kDecBlock = 1024;
constexpr int kDecWaves = kDecBlock / kWave;

// ---- block-wide reductions; `buf` has kDecWaves slots per value; every thread must call
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_add(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float block_max(float v, float* buf)
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    v = wave_max(v);
    __syncthreads();                                    // buf free again
    if (lane == 0) buf[wave] = v;
    __syncthreads();
    float r = buf[0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) r = fmaxf(r, buf[w]);
    return r;
}
__device__ __forceinline__ float block_add(float v, float* buf)
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    v = wave_add(v);
    __syncthreads();
    if (lane == 0) buf[wave] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) r += buf[w];    // fixed order
    return r;
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
template <bool kMin>
__device__ __forceinline__ void block_arg(float& v, int& i, float* fbuf, int* ibuf)
{
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(v, o);
        const int oi = __shfl_xor(i, o);
        if (better<kMin>(ov, oi, v, i)) { v = ov; i = oi; }
    }
    __syncthreads();
    if (lane == 0) { fbuf[wave] = v; ibuf[wave] = i; }
    __syncthreads();
    v = fbuf[0]; i = ibuf[0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w)
        if (better<kMin>(fbuf[w], ibuf[w], v, i)) { v = fbuf[w]; i = ibuf[w]; }
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
}

// (max, sum of 2^(x - max)) pairs of an online softmax; combine is associative
__device__ __forceinline__ void lse_combine(float& m, float& s, float om, float os)
{
    const float M = fmaxf(m, om);
    const float a = m > -INFINITY ? s * exp2_fast(m - M) : 0.f;
    const float b = om > -INFINITY ? os * exp2_fast(om - M) : 0.f;
    m = M;
    s = a + b;
}

// ------------------------------------------------------------------------------------
// Dynamic LDS (floats): dot[G][budget] | rn[budget] | en[n_imp] when that fits, else the
// same arrays live in the caller's workspace (a.lds_floats == 0).
template <typename T, int D, int G>
__global__ __launch_bounds__(kDecBlock) void decode_step_kernel(DecodeStepArgs a)
{
    using P = Pack<T>;
    constexpr int kE = P::kElems;
    constexpr int kLpr = Tile<T, D>::kChunksPerRow;          // lanes per cache row
    constexpr int kGroups = kDecBlock / kLpr;                // rows in flight per block

    extern __shared__ float dyn_lds[];
    __shared__ float fbuf[kDecWaves];
    __shared__ int ibuf[kDecWaves];
    __shared__ float vbuf[2 * G][kDecWaves];                 // vector reductions
    __shared__ float sh_self[G];                             // new query . new key (log2 units)
    __shared__ frag_t old_k[kLpr], old_v[kLpr];              // the token that leaves the window
    __shared__ float old_sc[4];                              // its norm, glo, past, cur
    __shared__ int old_pos;
    __shared__ float sh_newnorm;

    const int n_imp = a.n_imp, E = a.n_imp + a.n_tbm, W = a.window, Nb = a.budget;
    const int Tn = E + W;
    const int bkv = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
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
    const bool in_lds = a.lds_floats > 0;                    // block-uniform
    float* stage = in_lds ? dyn_lds : a.ws + (size_t)bkv * ((size_t)(G + 1) * Nb + n_imp);
    float* dot = stage;                                      // [G][budget] q_g . cache row
    float* rn_of = stage + (size_t)G * Nb;                   // [budget] copy of row_norm
    float* en = rn_of + Nb;                                  // [n_imp] norm of every stored entry key
    const char* qn = reinterpret_cast<const char*>(a.q_new) + (size_t)bkv * G * D * sizeof(T);
    const char* kn = reinterpret_cast<const char*>(a.k_new) + (size_t)bkv * D * sizeof(T);
    const char* vn = reinterpret_cast<const char*>(a.v_new) + (size_t)bkv * D * sizeof(T);

    // ---- phase 1: one dot product per cache row and q-head, the rows' own norms -------
    const int ct_mine = tid < n_imp ? entry_tok[tid] : 0;    // early: used in phase 4
    float qf[G][kE];
#pragma unroll
    for (int g = 0; g < G; ++g)
        P::unpack(*reinterpret_cast<const frag_t*>(qn + ((size_t)g * kLpr + piece) * 16), qf[g]);
    const frag_t new_k = *reinterpret_cast<const frag_t*>(kn + piece * 16);
    const frag_t new_v = *reinterpret_cast<const frag_t*>(vn + piece * 16);
    for (int r = tid; r < Nb; r += kDecBlock) rn_of[r] = row_norm[r];

    for (int r = grp; r < Nb + 1; r += kGroups) {
        // iteration r == Nb stands for the new token's own key
        const frag_t fk = r < Nb ? *reinterpret_cast<const frag_t*>(Kc + ((size_t)r * kLpr + piece) * 16) : new_k;
        float x[kE];
        P::unpack(fk, x);
        float d[G];
        float ss = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) d[g] = 0.f;
#pragma unroll
        for (int i = 0; i < kE; ++i) {
            ss = __builtin_fmaf(x[i], x[i], ss);
#pragma unroll
            for (int g = 0; g < G; ++g) d[g] = __builtin_fmaf(x[i], qf[g][i], d[g]);
        }
#pragma unroll
        for (int o = kLpr / 2; o >= 1; o >>= 1) {
            ss += __shfl_xor(ss, o);
#pragma unroll
            for (int g = 0; g < G; ++g) d[g] += __shfl_xor(d[g], o);
        }
        if (piece == 0) {
            if (r < Nb) {
#pragma unroll
                for (int g = 0; g < G; ++g) dot[(size_t)g * Nb + r] = d[g];
                if (r < n_imp) en[r] = sqrtf(ss);
            } else {
#pragma unroll
                for (int g = 0; g < G; ++g) sh_self[g] = a.scale_log2e * d[g];
                sh_newnorm = sqrtf(ss);
            }
        }
    }
    __syncthreads();

    // ---- phase 2: softmax over the live tokens and the new token (Eq. 1) ---------------
    // logit of token j in row r: scale * (|k_j| / |centre of r|) * (q . row r); one sweep
    // keeps a running (max, sum) per q-head, a second sweep forms the weights
    float m[G], sum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { m[g] = tid == 0 ? sh_self[g] : -INFINITY; sum[g] = tid == 0 ? 1.f : 0.f; }
    for (int j = tid; j < Tn; j += kDecBlock) {
        const int r = tok_row[j];
        if (r < 0) continue;
        const float rn = rn_of[r];
        const float c = a.scale_log2e * (rn > 0.f ? tok_norm[j] / rn : 0.f);
#pragma unroll
        for (int g = 0; g < G; ++g) lse_combine(m[g], sum[g], c * dot[(size_t)g * Nb + r], 1.f);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) lse_combine(m[g], sum[g], __shfl_xor(m[g], o), __shfl_xor(sum[g], o));
    }
    if (lane == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) { vbuf[2 * g][wave] = m[g]; vbuf[2 * g + 1][wave] = sum[g]; }
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = vbuf[2 * g][lane % kDecWaves];
        sum[g] = vbuf[2 * g + 1][lane % kDecWaves];
#pragma unroll
        for (int o = kDecWaves / 2; o >= 1; o >>= 1) lse_combine(m[g], sum[g], __shfl_xor(m[g], o), __shfl_xor(sum[g], o));
        sum[g] = 1.0f / sum[g];
    }
    // accumulate the row into s_Glo and s_Loc^cur (Sec. 3.2); the sums that Eq. 2 needs
    // (phase 4) are those of the updated scalars
    float sg = 0.f, sl = 0.f;
    for (int j = tid; j < Tn; j += kDecBlock) {
        const int r = tok_row[j];
        float w[G];
        if (r >= 0) {
            const float rn = rn_of[r];
            const float c = a.scale_log2e * (rn > 0.f ? tok_norm[j] / rn : 0.f);
            float tot = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) { w[g] = exp2_fast(c * dot[(size_t)g * Nb + r] - m[g]) * sum[g]; tot += w[g]; }
            const float glo = tok_glo[j] + tot, cur = tok_cur[j] + tot;
            tok_glo[j] = glo;
            tok_cur[j] = cur;
            sg += glo;
            sl += tok_past[j] + cur;
        } else {
#pragma unroll
            for (int g = 0; g < G; ++g) w[g] = 0.f;
        }
        if (a.attn_opt) {
#pragma unroll
            for (int g = 0; g < G; ++g) a.attn_opt[((size_t)bkv * G + g) * (Tn + 1) + j] = w[g];
        }
    }
    float self_tot = 0.f;                                    // every thread: same value
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float w = exp2_fast(sh_self[g] - m[g]) * sum[g];
        self_tot += w;
        if (a.attn_opt && tid == 0) a.attn_opt[((size_t)bkv * G + g) * (Tn + 1) + Tn] = w;
    }
    if (tid == 0) { sg += self_tot; sl += self_tot; }        // the new token: glo = cur = its own weight
    sg = wave_add(sg);
    sl = wave_add(sl);
    __syncthreads();                                         // vbuf free; every token's scalars written
    if (lane == 0) { vbuf[0][wave] = sg; vbuf[1][wave] = sl; }

    // ---- phase 3: the oldest window token leaves, the new token takes its ring slot ----
    const int ring = a.step % W;
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
        tok_pos[jo] = a.pos_new; tok_row[jo] = ro; tok_norm[jo] = sh_newnorm;
        tok_glo[jo] = self_tot; tok_past[jo] = 0.f; tok_cur[jo] = self_tot;
        row_norm[ro] = sh_newnorm;
    }
    __syncthreads();

    // ---- phase 4: least important class centre (Eq. 2 on the tokens' scalars) ----------
    sg = 0.f; sl = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) { sg += vbuf[0][w]; sl += vbuf[1][w]; }      // fixed order
    const float align = sg > 0.f ? sl / sg : 0.f;
    float bv = 0.f;
    int bi = -1;
    for (int s = tid; s < n_imp; s += kDecBlock) {
        const int ct = s == tid ? ct_mine : entry_tok[s];
        const float sc = fmaxf(tok_glo[ct] * align, tok_past[ct] + tok_cur[ct]);
        if (better<true>(sc, s, bv, bi)) { bv = sc; bi = s; }
    }
    block_arg<true>(bv, bi, fbuf, ibuf);
    const int s_star = max(bi, 0);                           // block-uniform, in [0, n_imp)
    const int f = entry_tok[s_star];

    // ---- phase 5: its most similar other centre (Eq. 5, cosine of the stored keys) -----
    float xs[kE];
    P::unpack(*reinterpret_cast<const frag_t*>(Kc + ((size_t)s_star * kLpr + piece) * 16), xs);
    const float en_star = en[s_star];
    const float rn_star = en_star > 0.f ? 1.0f / en_star : 0.f;
    float cv = 0.f;
    int ci = -1;
    for (int s = grp; s < n_imp; s += kGroups) {
        float x[kE];
        P::unpack(*reinterpret_cast<const frag_t*>(Kc + ((size_t)s * kLpr + piece) * 16), x);
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < kE; ++i) d = __builtin_fmaf(x[i], xs[i], d);
#pragma unroll
        for (int o = kLpr / 2; o >= 1; o >>= 1) d += __shfl_xor(d, o);
        const float e = en[s];
        const float sim = (d * (e > 0.f ? 1.0f / e : 0.f)) * rn_star;
        if (piece == 0 && s != s_star && better<false>(sim, s, cv, ci)) { cv = sim; ci = s; }
    }
    block_arg<false>(cv, ci, fbuf, ibuf);
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
    for (int j = tid; j < E; j += kDecBlock) {
        if (tok_row[j] != s_star || j == f) continue;
        if (merged) {
            tok_row[j] = dst;
        } else {
            tok_row[j] = -1; tok_pos[j] = -1;
            tok_norm[j] = 0.f; tok_glo[j] = 0.f; tok_past[j] = 0.f; tok_cur[j] = 0.f;
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

    // ---- phase 7: a full window of queries: s_Loc^cur becomes s_Loc^past (Sec. 3.2) ----
    if ((a.step + 1) % W == 0) {
        for (int j = tid; j < Tn; j += kDecBlock) { tok_past[j] = tok_cur[j]; tok_cur[j] = 0.f; }
    }
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

template <typename T, int D>
static hipError_t launch_decode_step_t(const DecodeStepArgs& a, hipStream_t st)
{
    const dim3 g(a.bkv), b(kDecBlock);
    const size_t lds = sizeof(float) * (size_t)a.lds_floats;
    switch (a.group) {
        case 1: hipLaunchKernelGGL((decode_step_kernel<T, D, 1>), g, b, lds, st, a); break;
        case 2: hipLaunchKernelGGL((decode_step_kernel<T, D, 2>), g, b, lds, st, a); break;
        case 4: hipLaunchKernelGGL((decode_step_kernel<T, D, 4>), g, b, lds, st, a); break;
        case 8: hipLaunchKernelGGL((decode_step_kernel<T, D, 8>), g, b, lds, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_decode_step(const DecodeStepArgs& a, bool f32, hipStream_t st)
{
    if (f32) return a.head_dim == 64 ? launch_decode_step_t<float, 64>(a, st) : launch_decode_step_t<float, 128>(a, st);
    return a.head_dim == 64 ? launch_decode_step_t<bf16_t, 64>(a, st) : launch_decode_step_t<bf16_t, 128>(a, st);
}

}  // namespace ems
