/*
 * ems_ref.h -- CPU oracle for the EMS prefill compression path (arXiv 2412.08521).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 implementation of what the
 * method computes, written from the paper.  It shares no code with the HIP library and
 * must never be used by a product path: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Every pointer is a HOST pointer.  Tensors are contiguous, row-major:
 *   q      [B, Hq , N, D]  float32 (bf16 inputs are widened exactly by the caller)
 *   k, v   [B, Hkv, N, D]  float32
 * q-head h reads kv-head h / (Hq/Hkv).
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py against
 * brute force, closed forms and invariants.  What the paper leaves open (GQA
 * aggregation, pooling padding, unweighted mean, placement of the zero-class row) is a
 * reading fixed by this build: parity is pinned given the reading, the reading itself
 * is "unpinned by the paper".
 */
#ifndef EMS_REF_H
#define EMS_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t batch;        /* B */
    int32_t q_heads;      /* Hq */
    int32_t kv_heads;     /* Hkv, divides Hq */
    int32_t head_dim;     /* D */
    int32_t seq_len;      /* N */
    int32_t window;       /* L_win: last-window queries / always-kept local tokens */
    int32_t budget;       /* N_budget = N_imp + L_win (Sec. 4.2) */
    int32_t pool_kernel;  /* odd mean-pool width, 1 = off (Sec. 4.2, Sec. 5.1) */
    double  merge_ratio;  /* r = gamma - 1 ; N_tbm = floor(r * N_budget) (Sec. 4.2) */
    double  tau;          /* merge iff similarity > tau (Sec. 4.2) */
    double  softmax_scale;/* <= 0 means 1/sqrt(D) (Eq. 1) */
} ems_ref_params;

/* N_imp = budget - window ; N_tbm = min(floor(r*budget), N - budget).  0 on success. */
int ems_ref_sizes(const ems_ref_params* p, int32_t* n_imp, int32_t* n_tbm);

/* Sec. 3.2: accumulated causal attention weights.  s_glo, s_loc are [B,Hkv,N] fp64,
 * summed over the q-heads of each kv group; lse_opt (nullable) is [B,Hq,N]. */
int ems_ref_score(const ems_ref_params* p, const float* q, const float* k,
                  double* s_glo, double* s_loc, double* lse_opt);

/* Eq. 2 followed by the mean pooling of Sec. 4.2.  s_out is [B,Hkv,N] fp64. */
int ems_ref_combine_pool(const ems_ref_params* p, const double* s_glo,
                         const double* s_loc, double* s_out);

/* Token partition of Sec. 4.2 on a given (pooled) score [B,Hkv,N]:
 * imp_idx [B,Hkv,N_imp], tbm_idx [B,Hkv,N_tbm], each ascending by position. */
int ems_ref_partition(const ems_ref_params* p, const double* s_pooled,
                      int32_t* imp_idx, int32_t* tbm_idx);

/* combine_pool + partition.  s_pooled_opt nullable. */
int ems_ref_select(const ems_ref_params* p, const double* s_glo, const double* s_loc,
                   double* s_pooled_opt, int32_t* imp_idx, int32_t* tbm_idx);

/* Eq. 5 with key-cosine similarity and threshold tau.
 * tbm_dest [B,Hkv,N_tbm]: slot in [0,N_imp) or `budget` for the zero class.
 * tbm_sim  [B,Hkv,N_tbm]: the winning similarity.
 * k_norm_opt (nullable) [B,Hkv,N_imp+N_tbm]: L2 norms of centre keys then TBM keys. */
int ems_ref_dest(const ems_ref_params* p, const float* k,
                 const int32_t* imp_idx, const int32_t* tbm_idx,
                 int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt);

/* Segmented average of Sec. 4.2 / App. A for given destinations.
 * k_out, v_out [B,Hkv,budget+1,D] fp64 (row `budget` = zero class),
 * kept_pos [B,Hkv,budget], slot_count [B,Hkv,N_imp+1] (last = zero class). */
int ems_ref_merge(const ems_ref_params* p, const float* k, const float* v,
                  const int32_t* imp_idx, const int32_t* tbm_idx,
                  const int32_t* tbm_dest,
                  double* k_out, double* v_out, int32_t* kept_pos, int32_t* slot_count);

/* dest + merge. */
int ems_ref_evict_merge(const ems_ref_params* p, const float* k, const float* v,
                        const int32_t* imp_idx, const int32_t* tbm_idx,
                        double* k_out, double* v_out, int32_t* kept_pos,
                        int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt,
                        int32_t* slot_count);

/* Eq. 5 with the redundancy of Sec. 4.1 / the similarity ablation of App. B:
 * similarity 0 = key cosine (same as ems_ref_dest), 1 = value cosine, 2 = their product.
 * k_norm_opt holds key norms in every mode. */
int ems_ref_dest_sim(const ems_ref_params* p, int similarity, const float* k, const float* v,
                     const int32_t* imp_idx, const int32_t* tbm_idx,
                     int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt);

/* Score-weighted merge (Sec. 4.2, last paragraph): as ems_ref_merge with every member
 * weighted by weight[pos] >= 0 ([B,Hkv,N] fp64; negatives count as 0).  An entry whose
 * weights add up to 0 keeps its centre; a zero class of total weight 0 is a zero row. */
int ems_ref_merge_weighted(const ems_ref_params* p, const float* k, const float* v,
                           const double* weight,
                           const int32_t* imp_idx, const int32_t* tbm_idx,
                           const int32_t* tbm_dest,
                           double* k_out, double* v_out, int32_t* kept_pos, int32_t* slot_count);

/* Eq. 3: sparsity rate per head from the Eq. 2 score (no pooling): 1 - N_k/N with N_k the
 * smallest number of top scores that reach zeta (0 < zeta <= 1) of the total.
 * p_out [B,Hkv]; n_k_opt [B,Hkv] nullable. */
int ems_ref_sparsity(const ems_ref_params* p, double zeta, const double* s_glo, const double* s_loc,
                     double* p_out, int32_t* n_k_opt);

/* Eq. 4: redundancy rate per head: share of tokens with an earlier token whose
 * key-cosine x value-cosine reaches tau.  r_out [B,Hkv]; best_opt [B,Hkv,N] nullable. */
int ems_ref_redundancy(const ems_ref_params* p, const float* k, const float* v,
                       double* r_out, double* best_opt);

/* The inner maximum of Eq. 4 for chosen tokens only: best_out [B,Hkv,n_tokens]. */
int ems_ref_redundancy_at(const ems_ref_params* p, const float* k, const float* v,
                          const int32_t* tokens, int32_t n_tokens, double* best_out);

/* Shared-entry expansion (App. A, "Shared Entry Expansion"; the position look-up-table of
 * Sec. 4.2): every kept token gets its run-time key and value back from its entry.
 * Row order per head: the N_imp centres, the N_tbm to-be-merged tokens (in tbm_idx order),
 * the L_win local tokens.  A token in entry s with key norm n gets key n * u_s, where
 * u_s = k_cache[s] / n_centre(s) is the entry's direction, and value v_cache[s]; tokens sent
 * to the zero class are evicted: zero row, position -1.
 *   k_cache, v_cache [B,Hkv,budget+1,D] fp64 ; kept_pos [B,Hkv,budget] ; tbm_idx, tbm_dest
 *   [B,Hkv,N_tbm] ; k_norm [B,Hkv,N_imp+N_tbm] (centres, then TBM tokens)
 *   k_exp, v_exp [B,Hkv,N_imp+N_tbm+L_win,D] fp64 ; pos_exp [B,Hkv,N_imp+N_tbm+L_win] */
int ems_ref_expand(const ems_ref_params* p, const double* k_cache, const double* v_cache,
                   const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
                   const double* k_norm, double* k_exp, double* v_exp, int32_t* pos_exp);

/* Number of OpenMP threads the score loop will use. */
int ems_ref_threads(void);

#ifdef __cplusplus
}
#endif
#endif
