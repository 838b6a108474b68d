/*
 * ems.h -- C ABI of the MI355X (gfx950) implementation of the EMS prefill compression
 * path (arXiv 2412.08521, "EMS: Adaptive Evict-then-Merge Strategy for Head-wise KV Cache
 * Compression Based on Global-Local Importance").
 *
 * One transformer layer's Q/K/V go in; a per-head Global-Local importance score, a token
 * partition and an equal-size compressed K/V cache come out.  Three calls, in order:
 *
 *     ems_global_local_score  ->  ems_select  ->  ems_evict_merge
 *
 * and, for the generation that follows, ems_expand (run-time keys/values of the compact
 * cache) and ems_decode_init -> ems_decode_step per generated token.
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer, contiguous and row-major, owned by the
 *     caller.  The library never allocates, frees or synchronises: work is enqueued on
 *     the caller's stream (`hip_stream` is a hipStream_t, NULL = the default stream) and
 *     scratch space comes in through `ws` (sizes from ems_workspace_bytes; 256-byte
 *     aligned; its contents need no initialisation and mean nothing between calls).
 *     ems_evict_merge_static is the one call without `ws`: it uses a fixed array that is
 *     part of the loaded library.  Outputs are fully overwritten.
 *   - Layouts (Appendix A, "Two-Levels of Parallelism": (batch, heads, len, head_dim)):
 *         q        [B, Hq , N, D]      k, v     [B, Hkv, N, D]
 *     in `dtype` (bf16 or f32).  q-head h attends kv-head h / (Hq/Hkv).
 *   - Return value: an ems_status.  Argument errors are found on the host before any
 *     launch; nothing is enqueued when a call fails with an argument error.
 *   - Calls that use the same workspace on different streams at once race.
 *
 * Derived sizes (Sec. 4.2): N_imp = budget - window class centres, N_tbm =
 * min(floor(merge_ratio * budget), N - budget) to-be-merged tokens, i.e. the paper's
 * merge magnification gamma = 1 + merge_ratio.  ems_partition_sizes returns them.
 */
#ifndef EMS_H
#define EMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EMS_OK = 0,
    EMS_ERR_INVALID_ARG = -1,  /* null pointer, inconsistent or out-of-range sizes */
    EMS_ERR_UNSUPPORTED = -2,  /* valid in principle, not built (e.g. head_dim) */
    EMS_ERR_WORKSPACE = -3,    /* ws is null, misaligned or smaller than required */
    EMS_ERR_LAUNCH = -4        /* the HIP runtime refused a launch */
} ems_status;

typedef enum {
    EMS_BF16 = 0,  /* bf16 I/O, bf16 MFMA with f32 accumulation */
    EMS_F32 = 1    /* f32 I/O, f32 MFMA: the validation mode */
} ems_dtype;

typedef enum {
    EMS_SIM_KEY = 0,       /* cosine of the keys */
    EMS_SIM_VALUE = 1,     /* cosine of the values */
    EMS_SIM_KEY_VALUE = 2  /* product of the two (the redundancy R of Sec. 4.1) */
} ems_similarity;

typedef struct {
    int32_t batch;         /* B  >= 1 */
    int32_t q_heads;       /* Hq >= 1 */
    int32_t kv_heads;      /* Hkv >= 1, divides Hq (grouped-query attention) */
    int32_t head_dim;      /* D in {64, 128} */
    int32_t seq_len;       /* N  >= 1 */
    int32_t window;        /* L_win: 1 <= window <= N; (< budget for select/evict_merge) */
    int32_t budget;        /* N_budget: window < budget <= N */
    float   merge_ratio;   /* r >= 0 : N_tbm = floor(r * budget), clamped to N - budget */
    float   tau;           /* merge iff cosine similarity > tau (paper: about 0.6) */
    int32_t pool_kernel;   /* odd >= 1 (<= 63) mean-pool width, 1 = off (paper: 7) */
    float   softmax_scale; /* <= 0 means 1/sqrt(D) (Eq. 1) */
    int32_t dtype;         /* ems_dtype of q, k, v, k_out, v_out */
} ems_params;

/* Library version (major*10000 + minor*100 + patch). */
int ems_version(void);

/* Static, human-readable text for an ems_status. */
const char* ems_strerror(int status);

/* Sec. 4.2 sizes: N_imp and N_tbm for these parameters (host only). */
int ems_partition_sizes(const ems_params* p, int32_t* n_imp, int32_t* n_tbm);

/* Bytes of device scratch each call needs for these parameters (host only; any of the
 * three outputs may be NULL). */
int ems_workspace_bytes(const ems_params* p, size_t* score_ws, size_t* select_ws,
                        size_t* merge_ws);

/*
 * Global and Local accumulated attention scores (Sec. 3.2; Eq. 1 gives the logits).
 * With A^h the N x N causal softmax attention matrix of q-head h (logits q_i.k_j * scale,
 * j <= i), per kv-head:
 *     s_glo[j] = sum_{h in group} sum_{i}            A^h[i][j]
 *     s_loc[j] = sum_{h in group} sum_{i >= N - window} A^h[i][j]
 * The N x N matrix is never stored: a first pass finds each row's log-sum-exp, a second
 * pass re-forms the weights tile by tile and adds them column-wise (App. A, "Global-Local
 * Score Efficiency Discussion").
 *   q, k      in : device, layouts above, `dtype`
 *   s_glo     out: device [B, Hkv, N] f32
 *   s_loc     out: device [B, Hkv, N] f32
 *   lse_opt   out: device [B, Hq, N] f32 natural-log row log-sum-exp, or NULL
 *   ws        device scratch of at least score_ws bytes
 * Uses batch, q_heads, kv_heads, head_dim, seq_len, window, softmax_scale, dtype.
 */
int ems_global_local_score(const ems_params* p, const void* q, const void* k,
                           float* s_glo, float* s_loc, float* lse_opt,
                           void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The two halves of ems_global_local_score as separate calls, for callers whose attention
 * kernel already produced the row log-sum-exp: the paper's own kernel re-uses that
 * "lse" of the forward pass and only re-forms the weights (App. A, "Global-Local Score
 * Efficiency Discussion").
 *   ems_attention_lse: lse[b][h][i] = ln sum_{j<=i} exp(q_i.k_j * scale), device
 *       [B, Hq, N] f32 (first pass only).
 *   ems_global_local_score_from_lse: s_glo / s_loc from q, k and such an lse (second pass
 *       only); with lse from ems_attention_lse the result equals ems_global_local_score
 *       up to the rounding of one ln/log2 conversion.
 * Workspace: score_ws bytes, as for ems_global_local_score.
 */
int ems_attention_lse(const ems_params* p, const void* q, const void* k, float* lse,
                      void* ws, size_t ws_bytes, void* hip_stream);
int ems_global_local_score_from_lse(const ems_params* p, const void* q, const void* k,
                                    const float* lse, float* s_glo, float* s_loc,
                                    void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Global-Local score (Eq. 2), mean pooling and token partition (Sec. 4.2).
 *     s[j]  = max( s_glo[j] * (sum(s_loc)/N) / (sum(s_glo)/N), s_loc[j] )
 *     s~[j] = (1/pool_kernel) * sum_{|t| <= (pool_kernel-1)/2} s[j+t]   (zeros outside)
 * The last `window` positions are local tokens and are not ranked.  Of the others, the
 * N_imp highest-scoring are the important tokens (class centres) and the next N_tbm the
 * to-be-merged tokens; equal scores rank by lower position first.
 *   s_glo, s_loc in : device [B, Hkv, N] f32
 *   s_gl_opt     out: device [B, Hkv, N] f32 pooled score s~ (all N positions), or NULL
 *   imp_idx      out: device [B, Hkv, N_imp] i32 positions, ascending
 *   tbm_idx      out: device [B, Hkv, N_tbm] i32 positions, ascending (may be NULL iff
 *                     N_tbm == 0)
 *   ws           device scratch of at least select_ws bytes
 */
int ems_select(const ems_params* p, const float* s_glo, const float* s_loc,
               float* s_gl_opt, int32_t* imp_idx, int32_t* tbm_idx,
               void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Head-wise evict-then-merge (Sec. 4.2, Eq. 5, App. A).  For every to-be-merged token i
 * the destination is d_i = argmax_c cos(k_i, k_c) over the class centres c (lowest slot on
 * ties); it merges into d_i if that similarity exceeds tau, else into the zero class
 * (eviction).  Every slot then holds the average of its members (the centre and the
 * tokens merged into it): values as a plain mean; keys as the mean of the members' unit
 * keys times the centre's own norm (the zero-class row keeps scale 1).  A slot nobody
 * joined is a bit-exact copy of its centre.  Rows N_imp..budget-1 are the `window` local
 * tokens, copied.  Every head therefore emits exactly `budget` cache rows plus one
 * zero-class row.
 *   k, v       in : device, layouts above, `dtype`
 *   imp_idx    in : device [B, Hkv, N_imp] i32, ascending, values in [0, N - window)
 *   tbm_idx    in : device [B, Hkv, N_tbm] i32 (NULL iff N_tbm == 0)
 *   k_out,v_out out: device [B, Hkv, budget + 1, D] `dtype`; row `budget` = zero class
 *                    (mean value / mean unit key of the evicted tokens, zeros if none)
 *   kept_pos   out: device [B, Hkv, budget] i32 source position of every cache row
 *   tbm_dest   out: device [B, Hkv, N_tbm] i32 slot in [0, N_imp) or `budget` (zero class)
 *   tbm_sim    out: device [B, Hkv, N_tbm] f32 winning cosine similarity
 *   k_norm_opt out: device [B, Hkv, N_imp + N_tbm] f32 key norms of centres, then of TBM
 *                    tokens, or NULL
 *   slot_count out: device [B, Hkv, N_imp + 1] i32 members per slot (last = zero class)
 *   ws         device scratch of at least merge_ws bytes
 * The index inputs are device data and cannot be checked on the host; positions outside
 * [0, N) are clamped into range by the kernels rather than dereferenced.
 */
int ems_evict_merge(const ems_params* p, const void* k, const void* v,
                    const int32_t* imp_idx, const int32_t* tbm_idx,
                    void* k_out, void* v_out, int32_t* kept_pos,
                    int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                    int32_t* slot_count,
                    void* ws, size_t ws_bytes, void* hip_stream);

/*
 * The paper-faithful variants of ems_evict_merge, same outputs and layouts:
 *   similarity        an ems_similarity: the redundancy R[i][d] that Eq. 5 maximises and tau
 *                     thresholds is the key cosine, the value cosine, or their product
 *                     (Sec. 4.1 "Redundancy"; similarity ablation of App. B).  A vector of norm 0
 *                     has cosine 0.  tbm_sim holds the winning R; k_norm holds key norms always.
 *   token_weight_opt  in : device [B, Hkv, N] f32, or NULL.  When given, the merge is weighted
 *                     by the tokens' attention scores (Sec. 4.2, last paragraph) -- e.g. the
 *                     pooled Global-Local score of ems_select: with w_i = max(weight, 0) of
 *                     member i (centre included), value = sum w_i v_i / sum w_i and key =
 *                     n_centre * sum w_i (k_i/|k_i|) / sum w_i.  An entry nobody joined, or whose
 *                     weights add up to 0, is a bit-exact copy of its centre; a zero class of
 *                     total weight 0 is a zero row.  slot_count still counts members.
 * With EMS_SIM_KEY and a NULL weight this is ems_evict_merge exactly.
 */
int ems_evict_merge_variant(const ems_params* p, int similarity, const void* k, const void* v,
                            const float* token_weight_opt,
                            const int32_t* imp_idx, const int32_t* tbm_idx,
                            void* k_out, void* v_out, int32_t* kept_pos,
                            int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                            int32_t* slot_count,
                            void* ws, size_t ws_bytes, void* hip_stream);

/*
 * ems_evict_merge for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, serving loops that hold no spare buffer, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and results as ems_evict_merge, minus `ws`:
 * the scratch is a fixed array of EMS_STATIC_SCRATCH_BYTES in each device's global memory
 * that belongs to the loaded library (held until the process ends).  The call allocates and
 * frees nothing.  The HIP device of `hip_stream` must be the current device.  The first call
 * on a device looks up that device's copy of the array (a HIP runtime query); make it once
 * outside any graph capture.
 *   returns EMS_ERR_WORKSPACE when the parameters need more than EMS_STATIC_SCRATCH_BYTES
 *   (merge_ws of ems_workspace_bytes), EMS_ERR_LAUNCH when the runtime refuses the look-up
 *   or a launch, otherwise as ems_evict_merge.
 * All calls on one device share that device's array and it keeps the last call's contents:
 * calls that overlap on one device (two streams, two host threads) race; serialise them.
 */
#define EMS_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
int ems_evict_merge_static(const ems_params* p, const void* k, const void* v,
                           const int32_t* imp_idx, const int32_t* tbm_idx,
                           void* k_out, void* v_out, int32_t* kept_pos,
                           int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                           int32_t* slot_count, void* hip_stream);

/*
 * Shared-entry expansion (App. A, "Shared Entry Expansion"; the position look-up-table of
 * Sec. 4.2).  Tokens that were merged share one cache entry; for the attention of the
 * current layer the compact cache is expanded back to one key / value per kept token.  The
 * look-up-table is what ems_evict_merge returned: tbm_dest (which entry each to-be-merged
 * token went to), kept_pos and k_norm (one key norm per token).  Rows per head, in order:
 * the N_imp centres, the N_tbm to-be-merged tokens (tbm_idx order), the `window` local
 * tokens -- N_exp = N_imp + N_tbm + window rows.  A token with key norm n in entry s gets
 * key (n / n_centre(s)) * k_cache[s] (the entry's direction times its own norm) and value
 * v_cache[s]; centres and local tokens are their own entries; tokens that went to the zero
 * class are evicted: zero rows with position -1, to be masked by the consumer.
 *   k_cache, v_cache in : device [B, Hkv, budget + 1, D] `dtype` (k_out / v_out of ems_evict_merge)
 *   kept_pos         in : device [B, Hkv, budget] i32
 *   tbm_idx, tbm_dest in: device [B, Hkv, N_tbm] i32 (NULL iff N_tbm == 0)
 *   k_norm           in : device [B, Hkv, N_imp + N_tbm] f32
 *   k_exp, v_exp     out: device [B, Hkv, N_exp, D] `dtype`
 *   pos_exp          out: device [B, Hkv, N_exp] i32 source position, -1 = evicted
 * No workspace.  Destinations outside [0, N_imp) are treated as the zero class.
 */
int ems_expand(const ems_params* p, const void* k_cache, const void* v_cache,
               const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
               const float* k_norm, void* k_exp, void* v_exp, int32_t* pos_exp,
               void* hip_stream);

/*
 * Per-head statistics of Sec. 4.1 (diagnostics: they motivate the method, the compression
 * itself does not need them).
 *
 * ems_sparsity_rate -- Eq. 3.  With s the Eq. 2 score of the head (ems_select's formula, no
 * pooling) sorted in descending order and N_k the smallest count whose leading scores add up
 * to at least zeta of the total, rate = 1 - N_k / N.
 *   zeta        0 < zeta <= 1
 *   s_glo, s_loc in : device [B, Hkv, N] f32
 *   rate        out: device [B, Hkv] f32
 *   n_k_opt     out: device [B, Hkv] i32, or NULL
 * Masses are compared in 40-bit fixed point relative to the total, so N_k can differ from an
 * exact evaluation where the threshold is met to within 1e-6 of the total.  No workspace.
 *
 * ems_redundancy_rate -- Eq. 4.  R[t][j] = cos(k_t, k_j) * cos(v_t, v_j); token t is redundant
 * if an EARLIER token j < t has R[t][j] >= tau; rate = redundant tokens / N.
 *   k, v        in : device [B, Hkv, N, D] `dtype`
 *   rate        out: device [B, Hkv] f32
 *   best        out: device [B, Hkv, N] f32: max over j < t of R[t][j] (-inf for t = 0)
 * O(N^2 D) work per head.  No workspace.  Uses tau, batch, kv_heads, head_dim, seq_len, dtype.
 */
int ems_sparsity_rate(const ems_params* p, float zeta, const float* s_glo, const float* s_loc,
                      float* rate, int32_t* n_k_opt, void* hip_stream);
int ems_redundancy_rate(const ems_params* p, const void* k, const void* v,
                        float* rate, float* best, void* hip_stream);

/*
 * Decode-time state of one layer's compressed cache (Sec. 3.3, decoding paragraph; Sec. 5
 * "Memory analysis": besides the budget-sized cache, one scalar per kept token for s_Glo,
 * s_Loc^past, s_Loc^cur, the key norm and the position look-up-table).  Every member is a
 * DEVICE pointer owned by the caller; T = N_imp + N_tbm + window tokens per head: the
 * look-up-table's N_imp + N_tbm elements (the centres first), then the window ring.
 *   k_cache, v_cache [B, Hkv, budget + 1, D] `dtype`: rows 0..N_imp-1 the entries, rows
 *                    N_imp..budget-1 the window ring (k_out / v_out of ems_evict_merge, updated
 *                    in place)
 *   row_norm    [B, Hkv, budget] f32  key norm of each row's centre token
 *   entry_count [B, Hkv, N_imp]  i32  tokens averaged into each entry
 *   entry_tok   [B, Hkv, N_imp]  i32  table index of each entry's centre token
 *   tok_pos     [B, Hkv, T] i32  position, -1 = free element
 *   tok_row     [B, Hkv, T] i32  cache row the token lives in, -1 = free element
 *   tok_norm, tok_glo, tok_past, tok_cur [B, Hkv, T] f32
 *   step_count  [1] i32  tokens generated so far (0 after ems_decode_init); lets a step be enqueued
 *                        without a host-side counter, e.g. from a captured HIP graph
 * A token's run-time key is (tok_norm / row_norm[row]) * k_cache[row], its value v_cache[row].
 */
typedef struct {
    void* k_cache;
    void* v_cache;
    float* row_norm;
    int32_t* entry_count;
    int32_t* entry_tok;
    int32_t* tok_pos;
    int32_t* tok_row;
    float* tok_norm;
    float* tok_glo;
    float* tok_past;
    float* tok_cur;
    int32_t* step_count;
} ems_decode_state;

/* Value of `step` that makes ems_decode_step read the counter in the state instead. */
#define EMS_STEP_FROM_STATE (-1)

/* Bytes of device scratch ems_decode_step needs (host only). */
int ems_decode_workspace_bytes(const ems_params* p, size_t* decode_ws);

/*
 * Fills the table and the scalars of `state` from what the prefill path returned (Sec. 3.3:
 * the prefill's s_Glo and s_Loc are stored for the generation; s_Loc is the first
 * s_Loc^past, s_Loc^cur starts at zero).  state->k_cache / v_cache must already hold
 * ems_evict_merge's k_out / v_out; they are read (window-row norms), not written.
 *   s_glo, s_loc in: device [B, Hkv, N] f32 (ems_global_local_score)
 *   kept_pos, tbm_dest, k_norm, slot_count in: ems_evict_merge's outputs; tbm_idx: ems_select's
 * To-be-merged tokens that went to the zero class get free table elements.
 */
int ems_decode_init(const ems_params* p, const float* s_glo, const float* s_loc,
                    const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
                    const float* k_norm, const int32_t* slot_count,
                    const ems_decode_state* state, void* hip_stream);

/*
 * One generated token (Sec. 3.3, decoding paragraph; App. A "Evict-then-Merge Details"),
 * for all heads in one launch.  `step` = number of tokens generated before this one, or
 * EMS_STEP_FROM_STATE to take it from state->step_count (a device scalar, so that the same
 * recorded launch can be replayed for token after token); either way step_count is left at
 * step + 1.  The new token's position is seq_len + step.  In order, per kv-head:
 *   1. attention row of the new queries (q-heads of the group, Eq. 1) over the run-time
 *      cache -- every live table element expanded, the window tokens, the new token itself;
 *   2. s_Glo and s_Loc^cur of every live token += the row (summed over the group);
 *   3. the oldest window token leaves the window; the new token takes its ring slot
 *      (row N_imp + step % window);
 *   4. the least important class centre -- Eq. 2 on its centre token's scalars, s_Loc =
 *      past + cur, alignment factor over all live tokens, lowest slot on ties -- becomes the
 *      single to-be-merged token;
 *   5. its destination is the other centre with the highest cosine of the stored entry keys
 *      (Eq. 5, lowest slot on ties); it merges iff that cosine exceeds tau, else it goes to
 *      the zero class (eviction);
 *   6. merge: the destination entry becomes the count-weighted mean of the two entries (values;
 *      unit-key means rescaled by the destination's centre norm) and the tokens that shared
 *      the departed entry now point to the destination; evict: their table elements are
 *      freed.  The token that left the window becomes the centre of the vacated entry and
 *      takes the departed centre's table element, so budget and table size stay constant;
 *   7. after every `window` steps s_Loc^past = s_Loc^cur, s_Loc^cur = 0.
 *   state        in/out
 *   q_new        in : device [B, Hq, D] `dtype`;  k_new, v_new in: device [B, Hkv, D] `dtype`
 *   attn_opt     out: device [B, Hq, T + 1] f32 attention weights (free elements 0, last =
 *                     the new token), or NULL
 *   decision_opt out: device [B, Hkv, 2] i32 (to-be-merged entry, destination or -1), or NULL
 *   sim_opt      out: device [B, Hkv] f32 the best cosine, or NULL
 *   ws           device scratch of at least decode_ws bytes
 * Supports Hq / Hkv in {1, 2, 4, 8}.  Steps on one state must be enqueued in order on one
 * stream.
 */
int ems_decode_step(const ems_params* p, const ems_decode_state* state, int32_t step,
                    const void* q_new, const void* k_new, const void* v_new,
                    float* attn_opt, int32_t* decision_opt, float* sim_opt,
                    void* ws, size_t ws_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EMS_H */
