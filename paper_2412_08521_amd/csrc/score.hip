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
// Both passes run one wave per work item, one wave per SIMD (the whole register file holds
// the stationary operand), with a private LDS ring for the streamed operand.
#include "ems_common.h"
#include "ems_kernels.h"

#include <type_traits>

namespace ems {

// ---- staging of the streamed operand: global memory -> LDS without passing through
// registers (global_load_lds_dwordx4), a ring of stages deep.
//
// One instruction moves 64 lanes x 16 bytes into 1 KiB of consecutive LDS; which 16 bytes of
// global memory a lane fetches is free, so rows are stored unpadded with their 16-byte
// chunks XOR-swizzled by the row number: the 16 lanes that read one chunk column of 16
// consecutive rows then hit 16 different bank groups.  Rows past the end of the matrix
// re-read the last row: callers never let such rows contribute (they are masked by
// causality or carry an infinite log-sum-exp).
template <typename T, int D>
__device__ __forceinline__ int swz_key(int row)
{
    return Tile<T, D>::kChunksPerRow >= 16 ? (row & 15) : ((row >> 1) & 7);
}

// One DMA instruction: every lane moves `kBytes` (16 or 4) from base + off (off per lane,
// base wave-uniform) to LDS byte address lds_addr + lane * kBytes (lds_addr wave-uniform;
// the hardware takes it from M0).  Written as inline assembly on purpose: the compiler would
// otherwise make every later LDS read wait for all DMA in flight, which defeats prefetching
// more than one stage ahead.  Completion is tracked by hand with wait_vmem().
template <int kBytes>
__device__ __forceinline__ void dma_to_lds(const void* base, unsigned off, unsigned lds_addr)
{
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_addr);
    if (kBytes == 16)
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(m0v) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(m0v) : "memory", "m0");
}

// Four 16-byte DMA instructions under one M0 value: the instruction's immediate offset
// (0, 1024, 2048, 3072) is added to the global address and to the LDS address alike, so
// instruction i moves 1 KiB from base + off_i + 1024 i to LDS lds_addr + 1024 i.  The
// per-lane offsets are passed without the 1024 i term; those of a stage's second (third, ..)
// group of four hold the group's 4 KiB instead, so that all groups share one base.
__device__ __forceinline__ void dma_to_lds_x4(const void* base, unsigned off0, unsigned off1, unsigned off2,
                                              unsigned off3, unsigned lds_addr)
{
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %5\n\t"
                 "global_load_lds_dwordx4 %0, %4\n\t"
                 "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
                 "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
                 "global_load_lds_dwordx4 %3, %4 offset:3072"
                 ::"v"(off0), "v"(off1), "v"(off2), "v"(off3), "s"(base), "s"(m0v) : "memory", "m0");
}

// The same two with the LDS address given as a wave-uniform base plus a compile-time offset: one
// scalar instruction sets M0.
template <int kLdsOff>
__device__ __forceinline__ void dma_to_lds_x4_at(const void* base, unsigned off0, unsigned off1, unsigned off2,
                                                 unsigned off3, unsigned lds_base)
{
    asm volatile("s_add_u32 m0, %5, %6\n\t"
                 "global_load_lds_dwordx4 %0, %4\n\t"
                 "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
                 "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
                 "global_load_lds_dwordx4 %3, %4 offset:3072"
                 ::"v"(off0), "v"(off1), "v"(off2), "v"(off3), "s"(base), "s"(lds_base), "n"(kLdsOff) : "memory", "m0", "scc");
}
template <int kLdsOff>
__device__ __forceinline__ void dma_dword_to_lds_at(const void* base, unsigned off, unsigned lds_base)
{
    asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_base), "n"(kLdsOff)
                 : "memory", "m0", "scc");
}

// The value itself, made opaque to the optimiser (stops loop-invariant code motion of what is
// computed from it).
__device__ __forceinline__ int opaque_lane(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// LDS byte address of a __shared__ object.
__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// Wait until at most kOutstanding of this wave's vector-memory operations are in flight
// (they complete in order), leaving the other counters alone.  The counts the kernels pass
// assume that between the DMA of a stage and its wait the wave issues NO other vector-memory
// instruction -- in particular no scratch (spill) load or store: the build rejects a score
// kernel whose compiled form uses scratch memory.
template <int kOutstanding>
__device__ __forceinline__ void wait_vmem()
{
    static_assert(kOutstanding >= 0 && kOutstanding < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kOutstanding) : "memory");
}

// The same wait for "nothing in flight", in the form the compiler can see: used once after
// the stationary operand's ordinary loads, so that the compiler does not re-insert a full
// wait for them in front of their first use inside the main loop.
__device__ __forceinline__ void wait_vmem_all_visible()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), expcnt and lgkmcnt left alone
}

// One wait for every LDS read in flight, in the form the compiler can see.  Placed well after a
// batch of fragment reads, it replaces the separate wait the compiler would otherwise put in
// front of each fragment's first use (a dozen scalar instructions per stage).
__device__ __forceinline__ void wait_lds_all_visible()
{
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), vmcnt and expcnt left alone
}

// The hardware deals workgroups to the 8 XCDs (each with its own L2) round-robin in launch
// order: block b runs on XCD b % 8.  First pass: work is cut into groups of `per_group`
// consecutive work items that stream the same operand; group g belongs to XCD g % 8 so that the
// group shares one L2.  Returns the linear index of the k-th work item of XCD `xcd`, or -1 for
// padding.
constexpr int kXcds = 8;
__device__ __forceinline__ int xcd_work_item(int n_groups, int per_group, int xcd, int k)
{
    const int group = (k / per_group) * kXcds + xcd;
    return group < n_groups ? group * per_group + k % per_group : -1;
}
static long long xcd_grid(long long n_groups, long long per_group)    // 8 x (items per XCD, padding included)
{
    return kXcds * ((n_groups + kXcds - 1) / kXcds) * per_group;
}

// ---- work queues.  The XCDs of one chip do not run at the same speed (a few percent apart under
// this load), and the hardware deals workgroups to them in fixed turns, so a launch whose work is
// bound to block indices ends when the slowest XCD ends, with the re-dispatch of a workgroup per
// item on top.  In long launches a wave therefore stays resident and takes its work items at run
// time, one integer atomic per item; which wave computes an item has no influence on the item's
// result.
// Second pass: from the queue of its XCD (items that stream the same operand stay on one L2)
// and, once that is empty, from a pool of the lightest items that every XCD draws from.  Returns
// the item's index in its queue (pool = true: in the pool), or -1 when both are empty.
__device__ __forceinline__ int take_work_item(int* cursors, int n_local, int n_pool, bool dynamic, bool& pool)
{
    if (!dynamic) {
        // short launches: one item per block, fixed by the block index (block b is the (b / 8)-th
        // of its XCD: first the XCD's queue, then every eighth item of the pool)
        const int x = blockIdx.x % kXcds, i = blockIdx.x / kXcds;
        pool = i >= n_local;
        const int k = pool ? (i - n_local) * kXcds + x : i;
        return pool && k >= n_pool ? -1 : k;
    }
    int k = -1, from_pool = 0;
    if (threadIdx.x == 0) {
        if (n_local > 0) {
            k = atomicAdd(&cursors[blockIdx.x % kXcds], 1);
            if (k >= n_local) k = -1;
        }
        if (k < 0 && n_pool > 0) {
            k = atomicAdd(&cursors[kXcds], 1);
            from_pool = 1;
            if (k >= n_pool) k = -1;
        }
    }
    pool = __builtin_amdgcn_readfirstlane(from_pool) != 0;
    return __builtin_amdgcn_readfirstlane(k);
}

// First pass: every XCD has a queue (its items in the fixed order of xcd_work_item, padding
// included); a wave whose own queue is empty goes on with the next item of another XCD's queue,
// so the faster XCDs help the slower ones finish.  Returns the item's index in the queue of XCD
// `from`, or -1 when every queue is empty.
__device__ __forceinline__ int take_or_steal(int* cursors, int n_per_queue, int& from)
{
    int k = -1, q = 0;
    if (threadIdx.x == 0) {
        const int own = blockIdx.x % kXcds;
        for (int d = 0; d < kXcds && k < 0; ++d) {
            q = (own + d) % kXcds;
            k = atomicAdd(&cursors[q], 1);
            if (k >= n_per_queue) k = -1;
        }
    }
    from = __builtin_amdgcn_readfirstlane(q);
    return __builtin_amdgcn_readfirstlane(k);
}

__global__ void score_queue_reset_kernel(int* queue)
{
    if (threadIdx.x < 2 * (kXcds + 1)) queue[threadIdx.x] = 0;      // both passes' cursors
}

// Pass 2: key tiles at or below the diagonal of row chunks 0..I, per (batch, kv-head): chunk I'
// has min(n_key_tiles, (I' + 1) * r) of them, r = chunk rows / keys per tile.
__host__ __device__ inline long long p2_items_upto(int I, int r, int n_key_tiles)
{
    const long long n = I + 1;
    const long long whole = n < n_key_tiles / r ? n : n_key_tiles / r;    // chunks whose count is not capped
    return r * whole * (whole + 1) / 2 + (n - whole) * n_key_tiles;
}

// sum of the 16 accumulator-derived values with four independent partial sums
__device__ __forceinline__ float sum16(const float (&p)[16])
{
    float s0 = p[0], s1 = p[1], s2 = p[2], s3 = p[3];
#pragma unroll
    for (int r = 4; r < 16; r += 4) { s0 += p[r]; s1 += p[r + 1]; s2 += p[r + 2]; s3 += p[r + 3]; }
    return (s0 + s1) + (s2 + s3);
}

__device__ __forceinline__ f32x16_t zero_acc()
{
    return f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
}

// One 32-key x 32-query tile of the online softmax.  kMasked tiles may cross the diagonal.
template <typename T, int D, bool kMasked>
__device__ __forceinline__ void pass1_tile(const frag_t (&ak)[Tile<T, D>::kFrags],
                                           const frag_t (&bq)[Tile<T, D>::kFrags],
                                           float& m_run, float& l_run, float c,
                                           int key0, int qi, int half)
{
    f32x16_t acc = zero_acc();
#pragma unroll
    for (int f = 0; f < Tile<T, D>::kFrags; ++f) mma<T>(acc, ak[f], bq[f]);
    if (kMasked) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (key0 + acc_row(r, half) > qi) acc[r] = -INFINITY;
    }
    float t0 = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
    float t1 = fmaxf(fmaxf(acc[3], acc[4]), acc[5]);
    float t2 = fmaxf(fmaxf(acc[6], acc[7]), acc[8]);
    float t3 = fmaxf(fmaxf(acc[9], acc[10]), acc[11]);
    float t4 = fmaxf(fmaxf(acc[12], acc[13]), acc[14]);
    t0 = fmaxf(fmaxf(t0, t1), t2);
    t3 = fmaxf(fmaxf(t3, t4), acc[15]);
    const float tmax = fmaxf(t0, t3);
    const float m_new = fmaxf(m_run, tmax * c);
    const float m_use = (kMasked && m_new == -INFINITY) ? 0.f : m_new;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = exp2_fast(__builtin_fmaf(acc[r], c, -m_use));
    l_run = __builtin_fmaf(l_run, exp2_fast(m_run - m_use), sum16(p));
    m_run = m_new;
}

// Combines the partial (max, sum) pairs of pass 1's key-range splits into the row
// log-sum-exp, in split order.
__global__ __launch_bounds__(256) void lse_combine_kernel(ScoreArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const size_t bh = blockIdx.y, BH = (size_t)a.batch * a.q_heads;
    if (i >= a.n_pad) return;
    float v = INFINITY;                                           // rows past the end: weight zero in pass 2
    if (i < a.seq_len) {
        float M = -INFINITY;
        for (int s = 0; s < a.p1_splits; ++s) M = fmaxf(M, a.part_m[((size_t)s * BH + bh) * a.n_pad + i]);
        float L = 0.f;
        for (int s = 0; s < a.p1_splits; ++s) {
            const float m = a.part_m[((size_t)s * BH + bh) * a.n_pad + i];
            if (m > -INFINITY) L += a.part_l[((size_t)s * BH + bh) * a.n_pad + i] * exp2_fast(m - M);
        }
        v = M + log2_fast(L);
        if (a.lse_opt) a.lse_opt[bh * a.seq_len + i] = v * 0.693147180559945309f;
    }
    a.lse2[bh * a.n_pad + i] = v;
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

// A caller's natural-log row log-sum-exp [B*Hq, N] -> the base-2, +inf-padded layout
// [B*Hq, n_pad] the second pass streams.
__global__ __launch_bounds__(256) void lse_to_base2_kernel(ScoreArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int bh = blockIdx.y;
    if (blockIdx.x == 0 && bh == 0 && threadIdx.x < 2 * (kXcds + 1)) a.queue[threadIdx.x] = 0;   // the pass that follows starts on empty queues
    if (i >= a.n_pad) return;
    a.lse2[(size_t)bh * a.n_pad + i] =
        i < a.seq_len ? a.lse_in_nat[(size_t)bh * a.seq_len + i] * 1.44269504088896340736f : INFINITY;
}


// ------------------------------------------------------------------------------------
// Pass 2, wave-private form.  A work item is ONE wave: it keeps 32 * kSub keys of one
// kv-head in registers (MFMA B operand, keys -> lanes) for its whole life and streams the
// query rows of one row chunk, 32 at a time, through an LDS ring that only this wave
// touches (DMA by this wave, read by this wave): no workgroup barrier anywhere.  One wave
// per SIMD owns the whole register file, so the stationary tile is large and every staged
// row is used for kSub MFMA tiles.
//
// The rows of a chunk fall in two classes, handled by two loops that share the ring:
//   edge rows      stages that touch the diagonal of this wave's keys or the last window:
//                  tiles are masked, skipped when above the diagonal, and (window rows) also
//                  added to the local score; a plain loop, one tile at a time;
//   interior rows  every row sees every key and no row is in the window: one software
//                  pipeline across tiles and stages.  Tiles go in pairs: the MFMA chains of
//                  the two tiles of a pair alternate (so consecutive matrix instructions never
//                  depend on each other) and between them the vector ALU turns the two
//                  accumulators the previous pair left behind into weights; the next stage's
//                  row operand and log-sum-exp are fetched from LDS into a second register set.
// 32-wide subtiles of the stationary operand per wave (8 x 8 fragments = the 256 accumulation
// registers in the 16-bit types) and LDS stages in the wave's ring
template <typename T> struct Stream { static constexpr int kSub = 8; static constexpr int kRing = 4; };
template <> struct Stream<float> { static constexpr int kSub = 2; static constexpr int kRing = 3; };
constexpr int kStreamRows = 32;            // query rows per stage (one MFMA row tile)
template <int v> using ic = std::integral_constant<int, v>;

// The interior loops' DMA cursor, one step: source address `q` advances by a stage (kQStep bytes), at
// the last stage of a head (h_left == 1 of per_head) by q_jump instead, and not at all once the
// last stage of all is issued (t_left <= 1); `l` likewise with kLStep / l_jump.  Written out: left
// to the compiler these few selects become several times as many instructions, part of them on
// the vector ALU.
template <int kQStep, int kLStep>
__device__ __forceinline__ void advance_cursor(int& h_left, int& t_left, const char*& q, const char*& l, int per_head,
                                               long long q_jump, long long l_jump)
{
    long long aq, al;
    asm volatile(
        "s_cmp_eq_u32 %[h], 1\n\t"
        "s_cselect_b64 %[aq], %[qj], %[qs]\n\t"
        "s_cselect_b64 %[al], %[lj], %[ls]\n\t"
        "s_cselect_b32 %[h], %[ph], %[h]\n\t"
        "s_sub_u32 %[h], %[h], 1\n\t"
        "s_cmp_gt_i32 %[t], 1\n\t"
        "s_cselect_b64 %[aq], %[aq], 0\n\t"
        "s_cselect_b64 %[al], %[al], 0\n\t"
        "s_sub_u32 %[t], %[t], 1"
        : [h] "+s"(h_left), [t] "+s"(t_left), [aq] "=&s"(aq), [al] "=&s"(al)
        : [qj] "s"(q_jump), [lj] "s"(l_jump), [ph] "s"(per_head + 1), [qs] "i"(kQStep), [ls] "i"(kLStep)
        : "scc");
    q += aq;
    l += al;
}

// The same for one source without heads (the first pass's keys).
template <int kStep>
__device__ __forceinline__ void advance_cursor(int& t_left, const char*& k)
{
    long long ak;
    asm volatile(
        "s_cmp_gt_i32 %[t], 1\n\t"
        "s_cselect_b64 %[ak], %[ks], 0\n\t"
        "s_sub_u32 %[t], %[t], 1"
        : [t] "+s"(t_left), [ak] "=&s"(ak)
        : [ks] "i"(kStep)
        : "scc");
    k += ak;
}


// One 32-row x 32-key tile of the edge loop: weights added into the lane's column sums; the
// tile may cross the diagonal and may hold last-window rows.
template <typename T, int D>
__device__ __forceinline__ void stream_edge_tile(const frag_t (&aq)[Tile<T, D>::kFrags],
                                                 const frag_t (&bk)[Tile<T, D>::kFrags],
                                                 const f32x16_t& lse_v, float c, float& glo, float& loc,
                                                 int row0, int kj, int half, int win0)
{
    constexpr int kFrags = Tile<T, D>::kFrags;
    f32x16_t acc = zero_acc();
    float p[16];
#pragma unroll
    for (int f = 0; f < kFrags; ++f) mma<T>(acc, aq[f], bk[f]);
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = exp2_fast(__builtin_fmaf(acc[r], c, -lse_v[r]));
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (row0 + acc_row(r, half) < kj) p[r] = 0.f;
    glo += sum16(p);
    if (row0 + 31 >= win0) {                               // wave-uniform
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (row0 + acc_row(r, half) < win0) p[r] = 0.f;
        loc += sum16(p);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(1, 1))) void score_pass2_stream_kernel(ScoreArgs a)
{
    constexpr int kSub = Stream<T>::kSub, kRing = Stream<T>::kRing;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kEps = 16 / kFrags;                       // accumulator elements handled per MFMA slot
    static_assert(kFrags >= 2 && kFrags <= 16 && 16 % kFrags == 0, "slot schedule needs 2..16 fragments per row");
    static_assert(kSub >= 2 && kSub % 2 == 0, "tiles are processed in pairs");
    constexpr int kPairs = kSub / 2;
    constexpr int kRowBytes = Tile<T, D>::kRowBytes;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kStageBytes = kStreamRows * kRowBytes;
    constexpr int kQInstr = kStageBytes / 1024;             // 16-byte DMA instructions per stage
    constexpr int kLoads = kQInstr + 1;                     // + one 4-byte DMA for the rows' log-sum-exp
    static_assert((kRing - 1) * kLoads < 64, "vmcnt is a 6-bit counter");
    static_assert(kRing == 3 || kRing == 4, "the waits below are written for rings of 3 or 4 stages");
    constexpr int kKeys = 32 * kSub;
    // stages per trip of the interior loop: after that many both the two operand register sets and
    // the ring slots are back where they started, so every slot is a compile-time constant
    constexpr int kUnroll = kRing % 2 ? 2 * kRing : kRing;

    __shared__ __attribute__((aligned(1024))) char lds_q[kRing][kStageBytes];
    __shared__ __attribute__((aligned(256))) float lds_lse[kRing][2 * kStreamRows];   // second half: spare

    const float c = a.scale_log2e;
    const int N = a.seq_len, W = a.window;
    const int G = a.q_heads / a.kv_heads;
    const int n_key_tiles = (N + kKeys - 1) / kKeys;
    const int n_chunks = a.n_chunks, R = a.chunk_rows;

    // Work item = (row chunk I, (batch, kv-head), key tile J at or below the chunk's diagonal),
    // heaviest chunks first.  An XCD's queue holds the chunks from the top down to p2_split for
    // its share of the heads (head = XCD + 8 m), key tiles innermost, so that the waves of an XCD
    // stream the same query rows; the chunks below p2_split, all heads, are the pool.
    const int BKV = a.batch * a.kv_heads;
    // Long launches: a wave stays and takes item after item until the queues are empty -- the exit
    // every wave reaches (the cursors only grow); between two items nothing of the wave is in flight.
    // Short launches: one item per block.
    // When the heads do not divide over the XCDs there are no queues: the groups (I, head) are
    // dealt to the XCDs in turn and every block has one item, fixed by its index.
    for (bool first = true; first || a.q_dynamic; first = false) {
    int I, J, bkv;
    if (a.q_share == 0) {
        int bid = xcd_work_item(BKV * n_chunks, n_key_tiles, blockIdx.x % kXcds, blockIdx.x / kXcds);
        if (bid < 0) break;
        J = bid % n_key_tiles; bid /= n_key_tiles;
        bkv = bid % BKV;
        I = n_chunks - 1 - bid / BKV;
    } else {
        bool pool;
        const int k = take_work_item(a.queue, a.p2_local, a.p2_pool, a.q_dynamic != 0, pool);
        if (k < 0) break;
        const int r_tiles = R / kKeys;
        const int top = pool ? a.p2_split - 1 : n_chunks - 1;
        const long long per = pool ? BKV : a.q_share;       // heads per chunk in this queue
        const long long upto_top = p2_items_upto(top, r_tiles, n_key_tiles);
        int lo = pool ? 0 : a.p2_split, hi = top;           // the chunk whose items include k: the smallest I with before(I) <= k
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (per * (upto_top - p2_items_upto(mid, r_tiles, n_key_tiles)) <= k) hi = mid; else lo = mid + 1;
        }
        I = lo;
        const int rem = (int)(k - per * (upto_top - p2_items_upto(I, r_tiles, n_key_tiles)));
        const int cnt = min(n_key_tiles, (I + 1) * r_tiles);
        J = rem % cnt;
        bkv = pool ? rem / cnt : (int)(blockIdx.x % kXcds) + kXcds * (rem / cnt);
    }
    const int key_base = J * kKeys;
    const int r_begin = max(I * R, key_base);               // both multiples of 32
    const int r_end = min((I + 1) * R, N);
    if (r_begin >= r_end) continue;                         // pair above the diagonal (the queues hold none)
    // [r_begin, e_end) touches the diagonal, [e_end, i_end) is interior, [i_end, r_end) holds
    // window rows (each range may be empty; all bounds but r_end are multiples of 32)
    const int win0 = N - W;
    int e_end = min(max(r_begin, min(key_base + kKeys, (win0 / kStreamRows) * kStreamRows)), r_end);
    const int i_end = min(max(e_end, (win0 / kStreamRows) * kStreamRows), r_end);
    // the interior loop takes kUnroll stages per trip: until their number divides, one more row
    // tile of every q-head goes to the edge loop (which is correct for any row)
    while ((((i_end - e_end) / kStreamRows) * G) % kUnroll) e_end += kStreamRows;

    const int b = bkv / a.kv_heads, kvh = bkv % a.kv_heads;
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;
    const T* Q0 = reinterpret_cast<const T*>(a.q) + ((size_t)(b * a.q_heads + kvh * G) * N) * D;
    const float* L0 = a.lse2 + (size_t)(b * a.q_heads + kvh * G) * a.n_pad;

    const int lane = threadIdx.x;
    const int col = lane & 31, half = lane >> 5;

    frag_t bk[kSub][kFrags];
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const int kj = key_base + s * 32 + col;
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            bk[s][f] = load_frag_or_zero(K, (size_t)kj * kRowBytes + f * 32 + half * 16, kj < N);
    }
    // The stationary operand lives in the accumulation registers, which only the matrix
    // instructions read: the ordinary vector registers stay free for what the ALU touches.
#pragma unroll
    for (int s = 0; s < kSub; ++s)
#pragma unroll
        for (int f = 0; f < kFrags; ++f) asm volatile("" : "+a"(bk[s][f]));

    // per-lane constants: DMA source offsets inside a stage (kept in registers when a stage is
    // few instructions; recomputed per stage otherwise, which only the wide-row validation
    // type needs) and the LDS offsets of this lane's operand fragments
    constexpr bool kKeepDmaOff = kQInstr <= 8;
    auto dma_src_off = [&](int j, int ln) __attribute__((always_inline)) {
        const int slot = j * kWave + ln, row = slot / kCpr;
        return (unsigned)row * kRowBytes + (unsigned)(((slot % kCpr) ^ swz_key<T, D>(row)) << 4);
    };
    unsigned dma_rel[kKeepDmaOff ? kQInstr : 1];            // the same, less the offset the instruction itself adds (1 KiB x its place in a group of four)
    if (kKeepDmaOff) {
#pragma unroll
        for (int j = 0; j < kQInstr; ++j) dma_rel[j] = dma_src_off(j, lane) - (unsigned)(j % 4) * 1024u;
    }
    unsigned frag_off[kFrags];
#pragma unroll
    for (int f = 0; f < kFrags; ++f)
        frag_off[f] = (unsigned)col * kRowBytes + (unsigned)(((f * 2 + half) ^ swz_key<T, D>(col)) << 4);

    const unsigned lds_q0 = lds_address(&lds_q[0][0]);
    const unsigned lds_l0 = lds_address(&lds_lse[0][0]);

    // DMA of the 32 rows starting at `row` of q-head g of the group into ring slot `slot`
    auto issue = [&](int g, int row, int slot, auto in_range_c) __attribute__((always_inline)) {
        constexpr bool kInRange = decltype(in_range_c)::value;   // caller knows row + 32 <= N
        const char* qg = reinterpret_cast<const char*>(Q0) + (size_t)g * N * kRowBytes;
        const unsigned dst = lds_q0 + slot * kStageBytes;
        int ln = lane;
        if (!kKeepDmaOff) ln = opaque_lane(ln);             // keeps the offsets from being hoisted into registers
        if (kInRange || row + kStreamRows <= N) {
            const char* base = qg + (size_t)row * kRowBytes;
            if (kKeepDmaOff && kQInstr % 4 == 0) {
#pragma unroll
                for (int j = 0; j < kQInstr; j += 4)
                    dma_to_lds_x4(base, dma_rel[j], dma_rel[j + 1], dma_rel[j + 2], dma_rel[j + 3], dst + j * 1024);
            } else {
#pragma unroll
                for (int j = 0; j < kQInstr; ++j)
                    dma_to_lds<16>(base, kKeepDmaOff ? dma_rel[j] + (unsigned)(j % 4) * 1024u : dma_src_off(j, ln), dst + j * 1024);
            }
        } else {                                            // rows past the end re-read the last row
#pragma unroll
            for (int j = 0; j < kQInstr; ++j) {
                const int r = (j * kWave + lane) / kCpr;
                const int over = max(row + r - (N - 1), 0);
                const unsigned off = kKeepDmaOff ? dma_rel[j] + (unsigned)(j % 4) * 1024u : dma_src_off(j, ln);
                dma_to_lds<16>(qg, (unsigned)row * kRowBytes + off - (unsigned)over * kRowBytes, dst + j * 1024);
            }
        }
        // the rows' log-sum-exp (padded with +inf up to n_pad); both half-waves fetch the same 32
        // values, the upper half into the spare half of the slot, so that no lane is masked off
        dma_to_lds<4>(L0 + (size_t)g * a.n_pad, (unsigned)(row + col) * 4u, lds_l0 + slot * (2 * kStreamRows * 4));
    };
    // with stages issued up to `last`, wait until stage t has landed (stages complete in order)
    auto wait_landed = [&](int t, int last) __attribute__((always_inline)) {
        const int later = last - t;
        if (later >= 2 && kRing > 3) wait_vmem<2 * kLoads>();
        else if (later >= 1) wait_vmem<kLoads>();
        else wait_vmem<0>();
    };
    // LDS -> registers: this lane's operand fragments of a staged row tile, and the 16 values of
    // the rows' log-sum-exp its accumulator registers stand for
    auto fetch_rows = [&](int slot, frag_t (&q_out)[kFrags], f32x16_t& l_out) __attribute__((always_inline)) {
        const char* qs = lds_q[slot];
        const float* ls = lds_lse[slot];
#pragma unroll
        for (int f = 0; f < kFrags; ++f) q_out[f] = *reinterpret_cast<const frag_t*>(qs + frag_off[f]);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(ls + 8 * q4 + 4 * half);
#pragma unroll
            for (int i = 0; i < 4; ++i) l_out[4 * q4 + i] = v[i];
        }
    };

    float part[kSub][kEps], loc[kSub];
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        loc[s] = 0.f;
#pragma unroll
        for (int e = 0; e < kEps; ++e) part[s][e] = 0.f;
    }

    wait_vmem_all_visible();

    // ---- edge rows: [r_begin, e_end) and [i_end, r_end) of every q-head of the group
    {
        const int lead = (e_end - r_begin) / kStreamRows;
        const int per_head = lead + (r_end - i_end + kStreamRows - 1) / kStreamRows;
        const int n_stages = per_head * G;
        auto row_of = [&](int t) __attribute__((always_inline)) {
            const int u = t % per_head;
            return u < lead ? r_begin + u * kStreamRows : i_end + (u - lead) * kStreamRows;
        };
        for (int t = 0; t < kRing - 1 && t < n_stages; ++t) issue(t / per_head, row_of(t), t % kRing, std::false_type{});
        for (int t = 0; t < n_stages; ++t) {
            if (t + kRing - 1 < n_stages)
                issue((t + kRing - 1) / per_head, row_of(t + kRing - 1), (t + kRing - 1) % kRing, std::false_type{});
            wait_landed(t, min(n_stages - 1, t + kRing - 1));
            frag_t aq[kFrags];
            f32x16_t lse_v;
            fetch_rows(t % kRing, aq, lse_v);
            const int row0 = row_of(t);
#pragma unroll
            for (int ks = 0; ks < kSub; ++ks) {
                const int ks0 = key_base + ks * 32;
                if (row0 + 31 >= ks0)                        // wave-uniform: not entirely above the diagonal
                    stream_edge_tile<T, D>(aq, bk[ks], lse_v, c, part[ks][0], loc[ks], row0, ks0 + col, half, win0);
                __builtin_amdgcn_sched_barrier(0);           // one tile's temporaries at a time
            }
            // the slot is re-filled by the DMA issued at the top of the next iteration: the
            // fragments above are in registers by then (their uses wait for them)
        }
        wait_vmem<0>();
    }

    // ---- interior rows: [e_end, i_end) of every q-head, one pipeline over all tiles.  The loop
    // body is straight-line code (an even number of stages, DMA issued for every stage index --
    // past the end the last stage is fetched again into a ring slot nobody reads -- and a constant
    // wait count), so nothing in it can be moved out of the slot it was written in.
    if (e_end < i_end) {
        const int per_head = (i_end - e_end) / kStreamRows;
        const int n_stages = per_head * G;                  // a multiple of kUnroll

        frag_t aq[2][kFrags];
        f32x16_t lse_v[2];
        f32x16_t acc[4];
        // issue cursor of the next stage to fetch: countdowns of the stages it has left in its q-head
        // and in all.  Where four DMA instructions go under one M0, the position is kept as running
        // addresses (source rows, their log-sum-exp) that advance by a stage, at the last stage of
        // a q-head by the jump to the next head's first interior row, and not at all once the last
        // stage is issued -- masks instead of selects, a dozen scalar instructions per stage.
        constexpr bool kRunning = kKeepDmaOff && kQInstr % 4 == 0;
        int h_left = per_head, t_left = n_stages;
        int g_next = 0, row_next = e_end;
        const char* q_src = reinterpret_cast<const char*>(Q0) + (size_t)e_end * kRowBytes;
        const char* l_src = reinterpret_cast<const char*>(L0 + e_end);
        const long long q_jump = ((long long)N - (i_end - e_end) + kStreamRows) * kRowBytes;   // last stage of a head -> next head
        const long long l_jump = ((long long)a.n_pad - (i_end - e_end) + kStreamRows) * 4;
        const unsigned lse_lane_off = (unsigned)col * 4u;
        const unsigned lds_q0s = __builtin_amdgcn_readfirstlane(lds_q0), lds_l0s = __builtin_amdgcn_readfirstlane(lds_l0);
        auto issue_next = [&](auto slot_c) __attribute__((always_inline)) {
            constexpr int slot = decltype(slot_c)::value;
            if constexpr (kRunning) {
                dma_to_lds_x4_at<slot * kStageBytes>(q_src, dma_rel[0], dma_rel[1], dma_rel[2], dma_rel[3], lds_q0s);
                if constexpr (kQInstr > 4)
                    dma_to_lds_x4_at<slot * kStageBytes + 4096>(q_src, dma_rel[4 % kQInstr], dma_rel[5 % kQInstr],
                                                                dma_rel[6 % kQInstr], dma_rel[7 % kQInstr], lds_q0s);
                static_assert(kQInstr <= 8 || !kRunning, "two groups of four per stage at most");
                dma_dword_to_lds_at<slot * (2 * kStreamRows * 4)>(l_src, lse_lane_off, lds_l0s);
                advance_cursor<kStageBytes, kStreamRows * 4>(h_left, t_left, q_src, l_src, per_head, q_jump, l_jump);
            } else {
                issue(g_next, row_next, slot, std::true_type{});
                const bool wrap = h_left == 1, more = t_left > 1;
                h_left = wrap ? per_head : h_left - 1;
                --t_left;
                g_next = more && wrap ? g_next + 1 : g_next;
                row_next = more ? (wrap ? e_end : row_next + kStreamRows) : row_next;
            }
        };

        issue_next(ic<0>{});
        issue_next(ic<1>{});
        if constexpr (kRing > 3) issue_next(ic<2>{});
        wait_vmem<(kRing - 2) * kLoads>();
        fetch_rows(0, aq[0], lse_v[0]);
        // Pairs alternate between accumulators {0, 1} and {2, 3}.  The pipeline starts on a pair
        // that weighs nothing: zero logits under an infinite log-sum-exp.
#pragma unroll
        for (int r = 0; r < 16; ++r) {                      // pair 0 of stage 0 writes {0, 1} and reads {2, 3}
            acc[2][r] = acc[3][r] = 0.f;
            lse_v[1][r] = INFINITY;
        }

        // One stage = kPairs rounds.  In round p the chains of tiles 2p and 2p+1 alternate, slot by
        // slot, and after each MFMA the vector ALU weighs kEps elements of the matching tile of the
        // previous pair (for p = 0 the last pair of the previous stage, whose rows' log-sum-exp is
        // in the other register set).  An accumulator is first read two MFMAs and a dozen vector
        // instructions after the chain that wrote it has ended.
        // the vector ALU's share of one MFMA slot: kEps accumulator elements turned into weights and
        // added to the column sums, written operation by operation so that no instruction follows
        // the one it depends on (the scheduler keeps this order where it does not interleave itself)
        auto weigh = [&](float (&sum)[kEps], const f32x16_t& s_acc, const f32x16_t& l, int f) __attribute__((always_inline)) {
            float x[kEps];
#pragma unroll
            for (int e = 0; e < kEps; ++e) x[e] = __builtin_fmaf(s_acc[f * kEps + e], c, -l[f * kEps + e]);
#pragma unroll
            for (int e = 0; e < kEps; ++e) x[e] = exp2_fast(x[e]);
#pragma unroll
            for (int e = 0; e < kEps; ++e) sum[e] += x[e];
        };
        auto stage = [&](auto u_c) __attribute__((always_inline)) {
            constexpr int u = decltype(u_c)::value;         // stage t of the trip, t = u (mod kUnroll)
            constexpr int set = u & 1;
            constexpr int kFetchAt = 1;                     // as early as the other register set is free: the LDS latency has three rounds to hide in
            issue_next(ic<(u + kRing - 1) % kRing>{});      // stage t + kRing - 1
#pragma unroll
            for (int p = 0; p < kPairs; ++p) {
                constexpr int kOddPairs = kPairs % 2;
                const int rp = (kOddPairs ? set + p : p) & 1;                 // accumulators this round writes: {2rp, 2rp+1}
                const int psa = (2 * p + kSub - 2) % kSub;                     // key subtiles of the previous pair
                f32x16_t& accA = acc[2 * rp];
                f32x16_t& accB = acc[2 * rp + 1];
                const f32x16_t& prevA = acc[2 * (1 - rp)];
                const f32x16_t& prevB = acc[2 * (1 - rp) + 1];
                const f32x16_t& pl = lse_v[p == 0 ? 1 - set : set];
#pragma unroll
                for (int f = 0; f < kFrags; ++f) {
                    if (f == 0) mma_first<T>(accA, aq[set][0], bk[2 * p][0]);
                    else mma<T>(accA, aq[set][f], bk[2 * p][f]);
                    weigh(part[psa], prevA, pl, f);
                    __builtin_amdgcn_sched_barrier(0);
                    if (f == 0) mma_first<T>(accB, aq[set][0], bk[2 * p + 1][0]);
                    else mma<T>(accB, aq[set][f], bk[2 * p + 1][f]);
                    weigh(part[psa + 1], prevB, pl, f);
                    // The other register set is free once round 0 has read the previous stage's
                    // log-sum-exp; stage t + 1 has landed once only the kRing - 2 stages issued
                    // after it are in flight.
                    if (kPairs > 1 && p == (kFetchAt < 1 ? 1 : kFetchAt) && f == 0) {
                        wait_vmem<(kRing - 2) * kLoads>();
                        fetch_rows((u + 1) % kRing, aq[1 - set], lse_v[1 - set]);
                    }
                    // two rounds later those reads have long returned: one wait for all of them
                    if (kPairs > 2 && kFetchAt < kPairs - 1 && p == kPairs - 1 && f == 0) wait_lds_all_visible();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (kPairs == 1) {                              // (validation type) nothing to hide the fetch behind
                wait_vmem<(kRing - 2) * kLoads>();
                fetch_rows((u + 1) % kRing, aq[1 - set], lse_v[1 - set]);
            }
        };
        for (int t = 0; t < n_stages; t += kUnroll) {
            stage(ic<0>{});
            stage(ic<1>{});
            stage(ic<2>{});
            stage(ic<3>{});
            if constexpr (kUnroll > 4) {
                stage(ic<4>{});
                stage(ic<5>{});
            }
        }
        // the last pair (key subtiles kSub - 2 and kSub - 1 of the last stage, register set 1)
        {
            constexpr int rp = ((kPairs % 2 ? 1 + kPairs - 1 : kPairs - 1)) & 1;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                part[kSub - 2][r % kEps] += exp2_fast(__builtin_fmaf(acc[2 * rp][r], c, -lse_v[1][r]));
                part[kSub - 1][r % kEps] += exp2_fast(__builtin_fmaf(acc[2 * rp + 1][r], c, -lse_v[1][r]));
            }
        }
        wait_vmem<0>();                                     // no DMA may outlive the wave's LDS
    }

    const int loc_chunk0 = a.loc_chunk0;
    float* out_glo = a.n_chunks == 1 ? a.s_glo + (size_t)bkv * N
                                     : a.part_glo + ((size_t)bkv * n_chunks + I) * N;
    float* out_loc = nullptr;
    if (a.n_chunks == 1) out_loc = a.s_loc + (size_t)bkv * N;
    else if (I >= loc_chunk0)
        out_loc = a.part_loc + ((size_t)bkv * (n_chunks - loc_chunk0) + (I - loc_chunk0)) * N;
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        float g = part[s][0];
#pragma unroll
        for (int e = 1; e < kEps; ++e) g += part[s][e];
        const float gsum = g + __shfl_xor(g, 32);           // the half-waves hold disjoint rows of the same keys
        const float lsum = loc[s] + __shfl_xor(loc[s], 32);
        const int kj = key_base + s * 32 + col;
        if (half == 0 && kj < N) {
            out_glo[kj] = gsum;
            if (out_loc) out_loc[kj] = lsum;
        }
    }
    }   // next work item
}

// ------------------------------------------------------------------------------------
// Pass 1, wave-private form.  A work item is ONE wave: it keeps 32 * kSub query rows of one
// q-head in registers (MFMA B operand, queries -> lanes) and streams the keys of its share of
// the causal range, 32 at a time, through its own LDS ring (A operand, keys -> accumulator
// registers): the row sum of a query is a per-lane scalar and there is no workgroup barrier.
//
//   online stages    the key stages that touch the diagonal of this wave's queries (masked),
//                    or, for a key range that has none, its first stage: textbook online
//                    softmax per tile (running maximum and rescaled sum), one tile at a time.
//                    They leave every lane a reference exponent m.
//   interior stages  every key is visible to every query: the software pipeline of the second
//                    pass (paired MFMA chains, weights of the previous pair in between), with
//                    the reference m held fixed: sum += exp2(c * S - m).  Any m gives the same
//                    log-sum-exp m + log2(sum) as long as the sum stays inside the float range,
//                    i.e. no later exponent exceeds m by ~100: if a sum does leave the range,
//                    the wave redoes its interior stages with the online form.
// ------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(1, 1))) void score_pass1_stream_kernel(ScoreArgs a)
{
    constexpr int kSub = Stream<T>::kSub, kRing = Stream<T>::kRing;
    constexpr int kFrags = Tile<T, D>::kFrags;
    constexpr int kEps = 16 / kFrags;
    static_assert(kFrags >= 2 && kFrags <= 16 && 16 % kFrags == 0, "slot schedule needs 2..16 fragments per row");
    static_assert(kSub >= 2 && kSub % 2 == 0, "tiles are processed in pairs");
    constexpr int kPairs = kSub / 2;
    constexpr int kRowBytes = Tile<T, D>::kRowBytes;
    constexpr int kCpr = Tile<T, D>::kChunksPerRow;
    constexpr int kStageBytes = kStreamRows * kRowBytes;
    constexpr int kLoads = kStageBytes / 1024;              // 16-byte DMA instructions per stage
    static_assert((kRing - 1) * kLoads < 64, "vmcnt is a 6-bit counter");
    static_assert(kRing == 3 || kRing == 4, "the waits below are written for rings of 3 or 4 stages");
    constexpr int kRows = 32 * kSub;                        // query rows per wave
    // stages per trip of the interior loop (operand register sets and ring slots back at their start)
    constexpr int kUnroll = kRing % 2 ? 2 * kRing : kRing;

    __shared__ __attribute__((aligned(1024))) char lds_k[kRing][kStageBytes];

    const int N = a.seq_len;
    const int n_row_tiles = (N + kRows - 1) / kRows;
    const int G = a.q_heads / a.kv_heads;
    // A wave stays and takes item after item until every queue is empty: the exit every wave
    // reaches (the cursors only grow); between two items nothing of the wave is in flight.
    // (Short launches: one item per block, by block index.)
    for (bool first = true; first || a.p1_dynamic; first = false) {
    int from_xcd = blockIdx.x % kXcds;
    const int k_item = a.p1_dynamic ? take_or_steal(a.queue + (kXcds + 1), a.p1_local, from_xcd) : (int)(blockIdx.x / kXcds);
    if (k_item < 0) break;
    int bid = xcd_work_item(a.p1_groups, a.p1_per_group, from_xcd, k_item);
    if (bid < 0) continue;                                  // padding
    const int S = a.p1_splits, sp = bid % S; bid /= S;           // this wave's share of the key range
    const int g = bid % G; bid /= G;
    const int BKV = a.batch * a.kv_heads;
    int rt, bkv;                                  // bkv = b * kv_heads + kv
    if (a.p1_groups == BKV) { rt = n_row_tiles - 1 - (bid % n_row_tiles); bkv = bid / n_row_tiles; }
    else { bkv = bid % BKV; rt = n_row_tiles - 1 - (bid / BKV); }   // heaviest row tiles first
    const int b = bkv / a.kv_heads, kvh = bkv % a.kv_heads;
    const int h = kvh * G + g;

    const T* Q = reinterpret_cast<const T*>(a.q) + ((size_t)(b * a.q_heads + h) * N) * D;
    const T* K = reinterpret_cast<const T*>(a.k) + ((size_t)bkv * N) * D;

    const int lane = threadIdx.x;
    const int col = lane & 31, half = lane >> 5;
    const int q_base = rt * kRows;
    const float c = a.scale_log2e;

    frag_t bq[kSub][kFrags];
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const int qi = q_base + s * 32 + col;
#pragma unroll
        for (int f = 0; f < kFrags; ++f)
            bq[s][f] = load_frag_or_zero(Q, (size_t)qi * kRowBytes + f * 32 + half * 16, qi < N);
    }
    // the stationary operand lives in the accumulation registers (only the matrix instructions read it)
#pragma unroll
    for (int s = 0; s < kSub; ++s)
#pragma unroll
        for (int f = 0; f < kFrags; ++f) asm volatile("" : "+a"(bq[s][f]));

    constexpr bool kKeepDmaOff = kLoads <= 8;
    auto dma_src_off = [&](int j, int ln) __attribute__((always_inline)) {
        const int slot = j * kWave + ln, row = slot / kCpr;
        return (unsigned)row * kRowBytes + (unsigned)(((slot % kCpr) ^ swz_key<T, D>(row)) << 4);
    };
    unsigned dma_rel[kKeepDmaOff ? kLoads : 1];             // less the offset the instruction itself adds (1 KiB x its place in a group of four)
    if (kKeepDmaOff) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) dma_rel[j] = dma_src_off(j, lane) - (unsigned)(j % 4) * 1024u;
    }
    unsigned frag_off[kFrags];
#pragma unroll
    for (int f = 0; f < kFrags; ++f)
        frag_off[f] = (unsigned)col * kRowBytes + (unsigned)(((f * 2 + half) ^ swz_key<T, D>(col)) << 4);
    const unsigned lds_k0 = lds_address(&lds_k[0][0]);

    // DMA of key stage t (keys 32 t ..) into ring slot `slot`
    auto issue = [&](int t, int slot, auto in_range_c) __attribute__((always_inline)) {
        constexpr bool kInRange = decltype(in_range_c)::value;   // caller knows 32 t + 32 <= N
        const int row = t * kStreamRows;
        const unsigned dst = lds_k0 + slot * kStageBytes;
        int ln = lane;
        if (!kKeepDmaOff) ln = opaque_lane(ln);
        if (kInRange || row + kStreamRows <= N) {
            const char* base = reinterpret_cast<const char*>(K) + (size_t)row * kRowBytes;
            if (kKeepDmaOff && kLoads % 4 == 0) {
#pragma unroll
                for (int j = 0; j < kLoads; j += 4)
                    dma_to_lds_x4(base, dma_rel[j], dma_rel[j + 1], dma_rel[j + 2], dma_rel[j + 3], dst + j * 1024);
            } else {
#pragma unroll
                for (int j = 0; j < kLoads; ++j)
                    dma_to_lds<16>(base, kKeepDmaOff ? dma_rel[j] + (unsigned)(j % 4) * 1024u : dma_src_off(j, ln), dst + j * 1024);
            }
        } else {                                            // keys past the end re-read the last key (always masked)
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                const int r = (j * kWave + lane) / kCpr;
                const int over = max(row + r - (N - 1), 0);
                const unsigned off = kKeepDmaOff ? dma_rel[j] + (unsigned)(j % 4) * 1024u : dma_src_off(j, ln);
                dma_to_lds<16>(K, (unsigned)row * kRowBytes + off - (unsigned)over * kRowBytes, dst + j * 1024);
            }
        }
    };
    auto wait_landed = [&](int t, int last) __attribute__((always_inline)) {
        const int later = last - t;
        if (later >= 2 && kRing > 3) wait_vmem<2 * kLoads>();
        else if (later >= 1) wait_vmem<kLoads>();
        else wait_vmem<0>();
    };
    auto fetch_keys = [&](int slot, frag_t (&k_out)[kFrags]) __attribute__((always_inline)) {
        const char* ks = lds_k[slot];
#pragma unroll
        for (int f = 0; f < kFrags; ++f) k_out[f] = *reinterpret_cast<const frag_t*>(ks + frag_off[f]);
    };

    // this wave's key stages: [t0, t1) of the stages a row tile can see; the stages from t_diag on
    // touch the diagonal
    const int last_key = min(N, q_base + kRows);                // exclusive
    const int n_all = (last_key + kStreamRows - 1) / kStreamRows;
    const int t0 = (int)((long long)n_all * sp / S), t1 = (int)((long long)n_all * (sp + 1) / S);
    const int t_diag = max(t0, q_base / kStreamRows);
    const int n_edge = max(t1 - t_diag, 0);
    // interior stages [t0, min(t1, t_diag)): the first n_lead of them are done in the online form --
    // one when there is no diagonal stage to take the reference from, more until the pipelined
    // rest is whole trips of the loop
    const int n_int_all = max(min(t1, t_diag) - t0, 0);
    int n_lead = n_edge == 0 && n_int_all > 0 ? 1 : 0;
    n_lead = __builtin_amdgcn_readfirstlane(n_lead + (n_int_all - n_lead) % kUnroll);   // (wave-uniform; kept in a scalar register)
    const int n_int = n_int_all - n_lead;                        // a multiple of kUnroll, >= 0

    float m_run[kSub], l_run[kSub];
#pragma unroll
    for (int s = 0; s < kSub; ++s) { m_run[s] = -INFINITY; l_run[s] = 0.f; }

    // Online form over a list of stages: `n_a` stages from `first_a`, then `n_b` from `first_b`.
    auto online_phase = [&](int first_a, int n_a, int first_b, int n_b) __attribute__((always_inline)) {
        const int n_stages = n_a + n_b;
        auto stage_of = [&](int u) __attribute__((always_inline)) { return u < n_a ? first_a + u : first_b + (u - n_a); };
        for (int u = 0; u < kRing - 1 && u < n_stages; ++u) issue(stage_of(u), u % kRing, std::false_type{});
        for (int u = 0; u < n_stages; ++u) {
            if (u + kRing - 1 < n_stages) issue(stage_of(u + kRing - 1), (u + kRing - 1) % kRing, std::false_type{});
            wait_landed(u, min(n_stages - 1, u + kRing - 1));
            frag_t ak[kFrags];
            fetch_keys(u % kRing, ak);
            const int key0 = stage_of(u) * kStreamRows;
#pragma unroll
            for (int s = 0; s < kSub; ++s) {
                const int qs0 = q_base + s * 32;
                if (key0 <= qs0 + 31)                        // wave-uniform: not entirely above the diagonal
                    pass1_tile<T, D, true>(ak, bq[s], m_run[s], l_run[s], c, key0, qs0 + col, half);
                __builtin_amdgcn_sched_barrier(0);           // one tile's temporaries at a time
            }
        }
        wait_vmem<0>();
    };

    wait_vmem_all_visible();
    online_phase(t0, n_lead, t_diag, n_edge);

    if (n_int > 0) {
        // A lane that has seen no key yet (its half of the diagonal tile lay above the diagonal)
        // borrows the reference of the other half of the wave, which holds the same queries.
        float m_fix[kSub], l_save[kSub];
#pragma unroll
        for (int s = 0; s < kSub; ++s) {
            const float m_o = __shfl_xor(m_run[s], 32);
            m_fix[s] = m_run[s] == -INFINITY ? (m_o == -INFINITY ? 0.f : m_o) : m_run[s];
            l_save[s] = l_run[s];
        }
        const int ti0 = t0 + n_lead;                             // interior stages [ti0, ti0 + n_int)

        frag_t ak[2][kFrags];
        f32x16_t acc[4];
        float lsum[kSub][kEps];
#pragma unroll
        for (int s = 0; s < kSub; ++s)
#pragma unroll
            for (int e = 0; e < kEps; ++e) lsum[s][e] = 0.f;

        // issue cursor: where four DMA instructions go under one M0, a running source address
        // that advances by a stage until the last stage is issued and then stays
        constexpr bool kRunning = kKeepDmaOff && kLoads % 4 == 0;
        int u_next = 0, t_left = n_int;
        const char* k_src = reinterpret_cast<const char*>(K) + (size_t)ti0 * kStageBytes;
        const unsigned lds_k0s = __builtin_amdgcn_readfirstlane(lds_k0);
        auto issue_next = [&](auto slot_c) __attribute__((always_inline)) {   // past the end: the last stage again, unread
            constexpr int slot = decltype(slot_c)::value;
            if constexpr (kRunning) {
                dma_to_lds_x4_at<slot * kStageBytes>(k_src, dma_rel[0], dma_rel[1], dma_rel[2], dma_rel[3], lds_k0s);
                if constexpr (kLoads > 4)
                    dma_to_lds_x4_at<slot * kStageBytes + 4096>(k_src, dma_rel[4 % kLoads], dma_rel[5 % kLoads],
                                                                dma_rel[6 % kLoads], dma_rel[7 % kLoads], lds_k0s);
                static_assert(kLoads <= 8 || !kRunning, "two groups of four per stage at most");
                advance_cursor<kStageBytes>(t_left, k_src);
            } else {
                issue(ti0 + min(u_next, n_int - 1), slot, std::true_type{});
                ++u_next;
            }
        };
        issue_next(ic<0>{});
        issue_next(ic<1>{});
        if constexpr (kRing > 3) issue_next(ic<2>{});
        wait_vmem<(kRing - 2) * kLoads>();
        fetch_keys(0, ak[0]);
        // the pipeline starts on a pair that weighs nothing: exponents of -inf
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[2][r] = acc[3][r] = -INFINITY;

        // One stage = kPairs rounds; in round p the chains of query subtiles 2p and 2p+1 alternate
        // and after each MFMA the vector ALU weighs kEps elements of the matching tile of the
        // previous pair (same structure as the second pass; the exponent's offset is the lane's m).
        // the vector ALU's share of one MFMA slot, operation by operation (no instruction follows
        // the one it depends on)
        auto weigh = [&](float (&sum)[kEps], const f32x16_t& s_acc, float m, int f) __attribute__((always_inline)) {
            float x[kEps];
#pragma unroll
            for (int e = 0; e < kEps; ++e) x[e] = __builtin_fmaf(s_acc[f * kEps + e], c, -m);
#pragma unroll
            for (int e = 0; e < kEps; ++e) x[e] = exp2_fast(x[e]);
#pragma unroll
            for (int e = 0; e < kEps; ++e) sum[e] += x[e];
        };
        auto stage = [&](auto u_c) __attribute__((always_inline)) {
            constexpr int u = decltype(u_c)::value;         // the stage's place in the trip
            constexpr int set = u & 1;
            issue_next(ic<(u + kRing - 1) % kRing>{});      // the stage kRing - 1 ahead
#pragma unroll
            for (int p = 0; p < kPairs; ++p) {
                constexpr int kOddPairs = kPairs % 2;
                const int rp = (kOddPairs ? set + p : p) & 1;
                const int psa = (2 * p + kSub - 2) % kSub;       // query subtiles of the previous pair
                f32x16_t& accA = acc[2 * rp];
                f32x16_t& accB = acc[2 * rp + 1];
                const f32x16_t& prevA = acc[2 * (1 - rp)];
                const f32x16_t& prevB = acc[2 * (1 - rp) + 1];
#pragma unroll
                for (int f = 0; f < kFrags; ++f) {
                    if (f == 0) mma_first<T>(accA, ak[set][0], bq[2 * p][0]);
                    else mma<T>(accA, ak[set][f], bq[2 * p][f]);
                    weigh(lsum[psa], prevA, m_fix[psa], f);
                    __builtin_amdgcn_sched_barrier(0);
                    if (f == 0) mma_first<T>(accB, ak[set][0], bq[2 * p + 1][0]);
                    else mma<T>(accB, ak[set][f], bq[2 * p + 1][f]);
                    weigh(lsum[psa + 1], prevB, m_fix[psa + 1], f);
                    if (kPairs > 1 && p == 1 && f == 0) {   // the other register set is free; early, so that the LDS latency hides
                        wait_vmem<(kRing - 2) * kLoads>();
                        fetch_keys((u + 1) % kRing, ak[1 - set]);
                    }
                    // two rounds later those reads have long returned: one wait for all of them
                    if (kPairs > 2 && p == kPairs - 1 && f == 0) wait_lds_all_visible();
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (kPairs == 1) {
                wait_vmem<(kRing - 2) * kLoads>();
                fetch_keys((u + 1) % kRing, ak[1 - set]);
            }
        };
        for (int u0 = 0; u0 < n_int; u0 += kUnroll) {
            stage(ic<0>{});
            stage(ic<1>{});
            stage(ic<2>{});
            stage(ic<3>{});
            if constexpr (kUnroll > 4) {
                stage(ic<4>{});
                stage(ic<5>{});
            }
        }
        {   // the last pair (query subtiles kSub - 2 and kSub - 1 of the last stage, register set 1)
            constexpr int rp = ((kPairs % 2 ? 1 + kPairs - 1 : kPairs - 1)) & 1;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                lsum[kSub - 2][r % kEps] += exp2_fast(__builtin_fmaf(acc[2 * rp][r], c, -m_fix[kSub - 2]));
                lsum[kSub - 1][r % kEps] += exp2_fast(__builtin_fmaf(acc[2 * rp + 1][r], c, -m_fix[kSub - 1]));
            }
        }
        wait_vmem<0>();

        // fold the interior sums into the running pair; a sum outside the float range (or NaN)
        // sends the whole wave back through its interior stages in the online form
        bool bad = false;
#pragma unroll
        for (int s = 0; s < kSub; ++s) {
            float t = lsum[s][0];
#pragma unroll
            for (int e = 1; e < kEps; ++e) t += lsum[s][e];
            // l_run is relative to m_run (or empty); rebase it to m_fix
            const float l_old = m_run[s] == -INFINITY ? 0.f : l_run[s];
            l_run[s] = l_old + t;
            m_run[s] = m_fix[s];
            bad |= !(l_run[s] < INFINITY);
        }
        if (__any(bad)) {
#pragma unroll
            for (int s = 0; s < kSub; ++s) {
                // back to the state after the first online phase (a lane that had seen a key has a
                // sum of at least one; an empty sum means the lane had no reference of its own)
                l_run[s] = l_save[s];
                m_run[s] = l_save[s] == 0.f ? -INFINITY : m_fix[s];
            }
            online_phase(ti0, n_int, 0, 0);
        }
    }

    const size_t bh = (size_t)(b * a.q_heads + h);
    float* lse2 = a.lse2 + bh * a.n_pad;
    float* lse_nat = a.lse_opt ? a.lse_opt + bh * N : nullptr;
#pragma unroll
    for (int s = 0; s < kSub; ++s) {
        const float m_o = __shfl_xor(m_run[s], 32);
        const float l_o = __shfl_xor(l_run[s], 32);
        const float M = fmaxf(m_run[s], m_o);
        const float Mu = (M == -INFINITY) ? 0.f : M;
        const float L = l_run[s] * exp2_fast(m_run[s] - Mu) + l_o * exp2_fast(m_o - Mu);
        const int qi = q_base + s * 32 + col;
        if (S > 1) {
            // partial (reference, sum) of this key range; combined by lse_combine_kernel
            if (half == 0 && qi < a.n_pad) {
                a.part_m[((size_t)sp * a.batch * a.q_heads + bh) * a.n_pad + qi] = M;
                a.part_l[((size_t)sp * a.batch * a.q_heads + bh) * a.n_pad + qi] = L;
            }
            continue;
        }
        const float v = Mu + log2_fast(L);
        // rows past the end get +inf: the second pass then gives them weight zero
        if (half == 0 && qi < a.n_pad) lse2[qi] = qi < N ? v : INFINITY;
        if (half == 0 && qi < N && lse_nat) lse_nat[qi] = v * 0.693147180559945309f;
    }
    }   // next work item
}

int score_keys_per_block(int dtype_is_f32) { return 32 * (dtype_is_f32 ? Stream<float>::kSub : Stream<bf16_t>::kSub); }

template <typename T, int D>
static hipError_t launch_pass1_t(ScoreArgs& a, hipStream_t st)
{
    constexpr int kRows = 32 * Stream<T>::kSub;
    const int BKV = a.batch * a.kv_heads, G = a.q_heads / a.kv_heads;
    const int n_row_tiles = (a.seq_len + kRows - 1) / kRows;
    // work items of one (b, kv-head) stream the same K: one group per XCD when there are enough
    // heads to keep all XCDs busy, else groups of the G q-heads of one row tile
    ScoreArgs a1 = a;
    const int S = a.p1_splits < 1 ? 1 : a.p1_splits;
    a1.p1_splits = S;
    if (BKV >= kXcds) { a1.p1_groups = BKV; a1.p1_per_group = n_row_tiles * G * S; }
    else { a1.p1_groups = BKV * n_row_tiles; a1.p1_per_group = G * S; }
    // one queue per XCD; resident waves, one per SIMD (128 per XCD) at most.  The reset (long
    // launches only: short ones do not use the cursors) clears the second pass's cursors as well.
    const long long per_xcd = xcd_grid(a1.p1_groups, a1.p1_per_group) / kXcds;
    if (kXcds * per_xcd > 0x7fffffffll) return hipErrorInvalidValue;
    a1.p1_local = (int)per_xcd;
    a1.p1_dynamic = per_xcd >= 4 * 128;                     // at least four rounds per resident wave
    const unsigned grid1 = (unsigned)(kXcds * (a1.p1_dynamic ? 128 : per_xcd));
    a.queue_clear = a1.p1_dynamic;                          // tells a second pass that follows whether it still has to clear its cursors
    if (a1.p1_dynamic) {
        hipLaunchKernelGGL(score_queue_reset_kernel, dim3(1), dim3(64), 0, st, a.queue);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    hipLaunchKernelGGL((score_pass1_stream_kernel<T, D>), dim3(grid1), dim3(kWave), 0, st, a1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    hipLaunchKernelGGL(lse_combine_kernel, dim3((a.n_pad + 255) / 256, a.batch * a.q_heads), dim3(256), 0, st, a1);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_pass2_t(const ScoreArgs& a, hipStream_t st)
{
    constexpr int kKeys = 32 * Stream<T>::kSub;
    const int BKV = a.batch * a.kv_heads;
    const int n_key_tiles = (a.seq_len + kKeys - 1) / kKeys;
    if (a.lse_in_nat) {
        dim3 g((a.n_pad + 255) / 256, a.batch * a.q_heads);
        hipLaunchKernelGGL(lse_to_base2_kernel, g, dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    // Queues: an XCD queue per share of the heads when they divide over the XCDs (else no queues:
    // groups dealt to the XCDs in turn, one block per pair).  With at least four rounds of items per resident wave (one wave per SIMD:
    // 128 per XCD) the waves stay and draw from the cursors, and the lightest row chunks -- about
    // 4.5 % of the items, which covers the spread between XCDs; more costs more in lost L2 sharing
    // than it balances -- go to the pool; shorter launches get one block per item.
    ScoreArgs a2 = a;
    const int r_tiles = a.chunk_rows / kKeys, top = a.n_chunks - 1;
    const long long all = p2_items_upto(top, r_tiles, n_key_tiles);
    a2.q_share = BKV % kXcds == 0 ? BKV / kXcds : 0;
    a2.q_dynamic = a2.q_share && (long long)BKV * all >= 4ll * 128 * kXcds;
    a2.p2_split = 0;
    if (a2.q_dynamic)
        while (a2.p2_split < top && p2_items_upto(a2.p2_split, r_tiles, n_key_tiles) <= all * 45 / 1000) ++a2.p2_split;
    const long long low = p2_items_upto(a2.p2_split - 1, r_tiles, n_key_tiles);
    const long long n_local = a2.q_share * (all - low), n_pool = (long long)BKV * low;
    const long long per_xcd = n_local + (n_pool + kXcds - 1) / kXcds;
    const long long grid2 = !a2.q_share ? xcd_grid((long long)BKV * a.n_chunks, n_key_tiles)     // no queues: a block per pair, padding included
                                        : kXcds * (a2.q_dynamic ? 128 : per_xcd);
    if (n_local > 0x7fffffffll || n_pool > 0x7fffffffll) return hipErrorInvalidValue;
    if (a.chunk_rows % kKeys != 0 || grid2 > 0x7fffffffll) return hipErrorInvalidValue;
    a2.p2_local = (int)n_local; a2.p2_pool = (int)n_pool;
    if (a2.q_dynamic && !a.lse_in_nat && !a.queue_clear) {  // (the conversion kernel above, or the first pass's launch, cleared them already)
        hipLaunchKernelGGL(score_queue_reset_kernel, dim3(1), dim3(64), 0, st, a.queue);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    }
    hipLaunchKernelGGL((score_pass2_stream_kernel<T, D>), dim3((unsigned)grid2), dim3(kWave), 0, st, a2);
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

hipError_t launch_score_pass1(ScoreArgs& a, bool f32, hipStream_t st) { EMS_DISPATCH(launch_pass1_t, a, f32, st); }
hipError_t launch_score_pass2(const ScoreArgs& a, bool f32, hipStream_t st) { EMS_DISPATCH(launch_pass2_t, a, f32, st); }

}  // namespace ems
