// Internal interface between the host-side C ABI (ems_api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ems {

struct ScoreArgs {
    const void* q;
    const void* k;
    float* s_glo;       // [B*Hkv, N]
    float* s_loc;       // [B*Hkv, N]
    float* lse_opt;     // [B*Hq, N] natural log, nullable
    float* lse2;        // [B*Hq, n_pad] base-2 log-sum-exp of c*S, +inf past N (workspace)
    const float* lse_in_nat;  // caller's natural-log row log-sum-exp for pass 2, or null
    float* part_glo;    // [B*Hkv, n_chunks, N] (workspace, n_chunks > 1 only)
    float* part_loc;    // [B*Hkv, n_chunks - loc_chunk0, N]
    int batch, q_heads, kv_heads, head_dim, seq_len, window;
    int n_pad;          // seq_len rounded up to a multiple of 64
    int n_chunks;       // row chunks of pass 2
    int chunk_rows;     // rows per chunk (multiple of 64)
    int loc_chunk0;     // first chunk that holds a last-window row
    float scale_log2e;  // softmax scale * log2(e)
    int p1_groups, p1_per_group;  // pass-1 work grouping per XCD (set by the launcher)
    int p1_splits;      // pass 1: key-range splits per row tile (1 = none)
    float* part_m;      // [p1_splits, B*Hq, n_pad] partial running maxima (workspace, p1_splits > 1)
    float* part_l;      // [p1_splits, B*Hq, n_pad] partial sums relative to them
    // Work queues (set by the launchers): a wave takes its work items from the queue of its XCD; once
    // that is empty, the first pass goes on with another XCD's queue, the second pass with a pool that
    // every XCD draws from.
    int* queue;         // [2][kXcds + 1] cursors: second pass, first pass (workspace; cleared before a pass)
    int p1_local;       // first pass: items per XCD queue
    int p1_dynamic;     // first pass: 1 = waves stay and draw (and steal), 0 = one item per block
    int queue_clear;    // the cursors are known to be clear (the pass follows the first pass's launch)
    int q_dynamic;      // 1: waves stay and take items from the cursors; 0: one item per block, by block index
    int q_share;        // (batch * kv_heads) / 8 heads per XCD queue; 0 = everything is in the pool
    int p2_split;       // row chunks below this index are in the pool
    int p2_local, p2_pool;   // items per XCD queue, items in the pool
};

struct SelectArgs {
    const float* s_glo;
    const float* s_loc;
    float* s_gl_opt;    // nullable
    float* pooled;      // [B*Hkv, N] workspace (pooled score = ranking keys; short sequences: Eq. 2 vector)
    // long sequences only (workspace):
    uint32_t* cand_key; // [B*Hkv, N] candidates' keys in integer order form, position order
    int32_t* cand_pos;  // [B*Hkv, N] their positions
    int* coarse_hist;   // [B*Hkv, select_coarse_bins()] keys per leading-bit bin
    float* chunk_sums;  // [B*Hkv, chunks, 2] sums of s_glo / s_loc per chunk
    int* chunk_count;   // [B*Hkv, chunks, 2] where a chunk's candidates start in the list, how many
    int* head_info;     // [B*Hkv] list cursor (ends as the length of the candidate list)
    int n_chunks;       // select_chunks(seq_len)
    int32_t* imp_idx;
    int32_t* tbm_idx;
    int bkv, seq_len, window, n_imp, n_tbm, pool_kernel;
};

struct MergeArgs {
    const void* k;
    const void* v;
    const int32_t* imp_idx;
    const int32_t* tbm_idx;
    void* k_out;
    void* v_out;
    int32_t* kept_pos;
    int32_t* tbm_dest;
    float* tbm_sim;
    float* k_norm;      // [B*Hkv, n_imp + n_tbm] (caller's k_norm_opt or workspace)
    int32_t* slot_count;
    int bkv, head_dim, seq_len, window, budget, n_imp, n_tbm;
    float tau;
    const float* weight;  // [B*Hkv, seq_len] per-token merge weight, or null = plain mean
    int similarity;       // 0 key cosine, 1 value cosine, 2 their product
    // centre slices of the destination search (dest_slicing); with one slice the partials are unused
    int slice_rows, n_slices;
    float* part_best;     // [B*Hkv, n_slices, n_tbm] best similarity within the slice
    int32_t* part_arg;    // [B*Hkv, n_slices, n_tbm] its centre
};

struct ExpandArgs {
    const void* k_cache;
    const void* v_cache;
    const int32_t* kept_pos;
    const int32_t* tbm_idx;
    const int32_t* tbm_dest;
    const float* k_norm;
    void* k_exp;
    void* v_exp;
    int32_t* pos_exp;
    int bkv, head_dim, window, budget, n_imp, n_tbm;
};

// Decode-time state of the compressed cache: one row per (batch, kv-head) in every array.
struct DecodeState {
    void* k_cache;          // [bkv, budget + 1, D]
    void* v_cache;
    float* row_norm;        // [bkv, budget]
    int32_t* entry_count;   // [bkv, n_imp]
    int32_t* entry_tok;     // [bkv, n_imp]
    int32_t* tok_pos;       // [bkv, T]   T = n_imp + n_tbm + window
    int32_t* tok_row;       // [bkv, T]   cache row, -1 = free element
    float* tok_norm;
    float* tok_glo;
    float* tok_past;
    float* tok_cur;
    int32_t* step_count;    // [1]
};

struct DecodeInitArgs {
    DecodeState st;
    const float* s_glo;     // [bkv, seq_len]
    const float* s_loc;
    const int32_t* kept_pos;
    const int32_t* tbm_idx;
    const int32_t* tbm_dest;
    const float* k_norm;
    const int32_t* slot_count;
    int bkv, head_dim, seq_len, window, budget, n_imp, n_tbm;
};

struct DecodeStepArgs {
    DecodeState st;
    const void* q_new;      // [bkv * group, D]
    const void* k_new;      // [bkv, D]
    const void* v_new;
    float* attn_opt;        // [bkv * group, T + 1] or null
    int32_t* decision_opt;  // [bkv, 2] or null
    float* sim_opt;         // [bkv] or null
    float* ws;              // [bkv, (group + 1) * budget] staging when it does not fit in LDS
    float* hand;            // [bkv, kDecodeHandFloats] hand-over record of the sliced step, else null
    int slice_rows, n_slices;   // row slices of the sliced step (decode_split); 0, 1 = one launch
    int lds_floats;         // (group + 1) * budget when staged in LDS, else 0
    int bkv, group, head_dim, seq_len, window, budget, n_imp, n_tbm;
    int step;               // >= 0, or -1: read st.step_count
    float tau, scale_log2e;
};

struct StatsArgs {
    const float* s_glo;     // [bkv, seq_len]   (sparsity)
    const float* s_loc;
    float* p_out;           // [bkv]
    int32_t* n_k_opt;       // [bkv] or null
    const void* k;          // [bkv, seq_len, D] (redundancy)
    const void* v;
    float* r_out;           // [bkv]
    float* best;            // [bkv, seq_len]
    int bkv, head_dim, seq_len;
    float zeta, tau;
};

int score_keys_per_block(int dtype_is_f32);
int select_chunks(int seq_len);     // blocks per head of the long-sequence select
int select_coarse_bins();
hipError_t launch_sparsity(const StatsArgs& a, hipStream_t st);
hipError_t launch_redundancy(const StatsArgs& a, bool f32, hipStream_t st);
hipError_t launch_decode_init(const DecodeInitArgs& a, bool f32, hipStream_t st);
hipError_t launch_decode_step(const DecodeStepArgs& a, bool f32, hipStream_t st);
constexpr int kDecodeMaxSlices = 32;     // row slices per head of the sliced decode step
constexpr int kDecodeHandFloats = 384;   // floats of its per-head hand-over record
bool decode_split(int budget, int n_imp, int n_tbm, int window, bool f32, int* slice_rows, int* n_slices);
hipError_t launch_expand(const ExpandArgs& a, bool f32, hipStream_t st);
hipError_t launch_score_pass1(ScoreArgs& a, bool f32, hipStream_t st);   // rows' log-sum-exp; sets a.queue_clear
hipError_t launch_score_pass2(const ScoreArgs& a, bool f32, hipStream_t st);   // column sums
hipError_t launch_select(const SelectArgs& a, hipStream_t st);
hipError_t launch_evict_merge(const MergeArgs& a, bool f32, hipStream_t st);
void dest_slicing(int n_imp, bool f32, int* slice_rows, int* n_slices);

}  // namespace ems
