/*
 * ems_ref.c -- CPU oracle for the EMS prefill compression path (arXiv 2412.08521).
 *
 * TEST INFRASTRUCTURE ONLY (see ems_ref.h).  Plain loops, fp64 throughout, no tiling,
 * no fusion: every function takes the steps of the paper in the paper's order so that
 * it can be checked against the text by eye.  OpenMP only spreads independent rows /
 * heads over cores.
 */
#include "ems_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_BAD (-1)

static int score_params_ok(const ems_ref_params* p)
{
    if (!p) return 0;
    if (p->batch < 1 || p->q_heads < 1 || p->kv_heads < 1 || p->head_dim < 1) return 0;
    if (p->q_heads % p->kv_heads) return 0;
    if (p->seq_len < 1 || p->window < 1 || p->window > p->seq_len) return 0;
    return 1;
}

static int full_params_ok(const ems_ref_params* p)
{
    if (!score_params_ok(p)) return 0;
    if (!(p->window < p->budget && p->budget <= p->seq_len)) return 0;
    if (p->pool_kernel < 1 || (p->pool_kernel % 2) == 0) return 0;
    if (!(p->merge_ratio >= 0.0)) return 0;
    return 1;
}

int ems_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sec. 4.2: N_budget = N_imp + L_win ; gamma = (N_budget + N_tbm) / N_budget, so with
 * r = gamma - 1 the to-be-merged set holds floor(r * N_budget) tokens, limited by the
 * number of candidates that are neither local nor important. */
int ems_ref_sizes(const ems_ref_params* p, int32_t* n_imp, int32_t* n_tbm)
{
    if (!full_params_ok(p)) return REF_BAD;
    int32_t imp = p->budget - p->window;
    double want = floor(p->merge_ratio * (double)p->budget);
    int32_t room = p->seq_len - p->budget; /* = N - W - N_imp */
    int32_t tbm = want > (double)room ? room : (int32_t)want;
    if (n_imp) *n_imp = imp;
    if (n_tbm) *n_tbm = tbm;
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Sec. 3.2.  A is the N x N causal attention weight matrix of one q-head:
 *   A[i][j] = softmax_j( q_i . k_j / sqrt(D) ), j <= i        (Eq. 1 gives the scale)
 *   s_Glo = sum over all rows i of A[i][:]
 *   s_Loc = sum over the last L_win rows of A[i][:]
 * With grouped-query attention the q-heads of a group are added into their kv-head.
 * ---------------------------------------------------------------------------------- */
int ems_ref_score(const ems_ref_params* p, const float* q, const float* k,
                  double* s_glo, double* s_loc, double* lse_opt)
{
    if (!score_params_ok(p) || !q || !k || !s_glo || !s_loc) return REF_BAD;
    const long B = p->batch, Hq = p->q_heads, Hkv = p->kv_heads, D = p->head_dim;
    const long N = p->seq_len, W = p->window, G = Hq / Hkv;
    const double scale = p->softmax_scale > 0.0 ? p->softmax_scale : 1.0 / sqrt((double)D);

    memset(s_glo, 0, sizeof(double) * (size_t)(B * Hkv * N));
    memset(s_loc, 0, sizeof(double) * (size_t)(B * Hkv * N));

    const int T = ems_ref_threads();
    double* part = (double*)malloc(sizeof(double) * (size_t)T * 2 * (size_t)N);
    double* rows = (double*)malloc(sizeof(double) * (size_t)T * (size_t)N);
    double* kd = (double*)malloc(sizeof(double) * (size_t)(N * D));
    if (!part || !rows || !kd) { free(part); free(rows); free(kd); return REF_BAD; }

    for (long b = 0; b < B; ++b) {
        for (long h = 0; h < Hq; ++h) {
            const long kv = h / G;
            const float* Qh = q + ((b * Hq + h) * N) * D;
            const float* Kh = k + ((b * Hkv + kv) * N) * D;
            double* glo = s_glo + (b * Hkv + kv) * N;
            double* loc = s_loc + (b * Hkv + kv) * N;
            double* lse = lse_opt ? lse_opt + (b * Hq + h) * N : NULL;
            for (long t = 0; t < N * D; ++t) kd[t] = (double)Kh[t];
            memset(part, 0, sizeof(double) * (size_t)T * 2 * (size_t)N);

#pragma omp parallel num_threads(T)
            {
#ifdef _OPENMP
                const int tid = omp_get_thread_num();
#else
                const int tid = 0;
#endif
                double* a = rows + (size_t)tid * (size_t)N;
                double* pg = part + (size_t)tid * 2 * (size_t)N;
                double* pl = pg + N;
                double qd[1024];
                double* qbuf = D <= 1024 ? qd : (double*)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(static, 1)
                for (long i = 0; i < N; ++i) {
                    for (long d = 0; d < D; ++d) qbuf[d] = (double)Qh[i * D + d];
                    double m = -INFINITY;
                    for (long j = 0; j <= i; ++j) {
                        const double* kj = kd + j * D;
                        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
                        for (long d = 0; d < D; ++d) acc += qbuf[d] * kj[d];
                        a[j] = acc * scale;
                        if (a[j] > m) m = a[j];
                    }
                    double sum = 0.0;
                    for (long j = 0; j <= i; ++j) { a[j] = exp(a[j] - m); sum += a[j]; }
                    const int local_row = (i >= N - W);
                    for (long j = 0; j <= i; ++j) {
                        const double w = a[j] / sum;
                        pg[j] += w;
                        if (local_row) pl[j] += w;
                    }
                    if (lse) lse[i] = m + log(sum);
                }
                if (qbuf != qd) free(qbuf);
            }
            /* fixed-order reduction over threads */
            for (int t = 0; t < T; ++t) {
                const double* pg = part + (size_t)t * 2 * (size_t)N;
                const double* pl = pg + N;
                for (long j = 0; j < N; ++j) { glo[j] += pg[j]; loc[j] += pl[j]; }
            }
        }
    }
    free(part); free(rows); free(kd);
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Eq. 2: s = max( s_Glo * (sum(s_Loc)/N) / (sum(s_Glo)/N) , s_Loc ) element-wise,
 * then the mean pooling of Sec. 4.2 (stride 1, same length, zero padding, divisor
 * always the kernel width).
 * ---------------------------------------------------------------------------------- */
int ems_ref_combine_pool(const ems_ref_params* p, const double* s_glo,
                         const double* s_loc, double* s_out)
{
    if (!score_params_ok(p) || !s_glo || !s_loc || !s_out) return REF_BAD;
    if (p->pool_kernel < 1 || (p->pool_kernel % 2) == 0) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len;
    const long half = (p->pool_kernel - 1) / 2;
    double* s = (double*)malloc(sizeof(double) * (size_t)N);
    if (!s) return REF_BAD;
    for (long u = 0; u < BH; ++u) {
        const double* glo = s_glo + u * N;
        const double* loc = s_loc + u * N;
        double sum_glo = 0.0, sum_loc = 0.0;
        for (long j = 0; j < N; ++j) { sum_glo += glo[j]; sum_loc += loc[j]; }
        const double align = (sum_loc / (double)N) / (sum_glo / (double)N);
        for (long j = 0; j < N; ++j) {
            const double g = glo[j] * align;
            s[j] = g > loc[j] ? g : loc[j];
        }
        for (long j = 0; j < N; ++j) {
            double acc = 0.0;
            for (long t = -half; t <= half; ++t) {
                const long jj = j + t;
                if (jj >= 0 && jj < N) acc += s[jj];
            }
            s_out[u * N + j] = acc / (double)p->pool_kernel;
        }
    }
    free(s);
    return REF_OK;
}

typedef struct { double score; int32_t pos; } ranked_t;

/* higher score first; equal scores: lower position first */
static int by_rank(const void* x, const void* y)
{
    const ranked_t* a = (const ranked_t*)x;
    const ranked_t* b = (const ranked_t*)y;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->pos > b->pos) - (a->pos < b->pos);
}

static int by_pos(const void* x, const void* y)
{
    const int32_t a = *(const int32_t*)x, b = *(const int32_t*)y;
    return (a > b) - (a < b);
}

/* ------------------------------------------------------------------------------------
 * Sec. 4.2, token partition.  The last L_win tokens are local and always kept; the
 * others are ranked by score: the first N_imp are the important tokens (class
 * centres), the next N_tbm the to-be-merged tokens, the rest irrelevant (evicted).
 * ---------------------------------------------------------------------------------- */
int ems_ref_partition(const ems_ref_params* p, const double* s_pooled,
                      int32_t* imp_idx, int32_t* tbm_idx)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK || !s_pooled || !imp_idx) return REF_BAD;
    if (n_tbm > 0 && !tbm_idx) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len;
    const long cand = N - p->window;
    ranked_t* r = (ranked_t*)malloc(sizeof(ranked_t) * (size_t)(cand > 0 ? cand : 1));
    if (!r) return REF_BAD;
    for (long u = 0; u < BH; ++u) {
        for (long j = 0; j < cand; ++j) { r[j].score = s_pooled[u * N + j]; r[j].pos = (int32_t)j; }
        qsort(r, (size_t)cand, sizeof(ranked_t), by_rank);
        for (long t = 0; t < n_imp; ++t) imp_idx[u * n_imp + t] = r[t].pos;
        for (long t = 0; t < n_tbm; ++t) tbm_idx[u * n_tbm + t] = r[n_imp + t].pos;
        qsort(imp_idx + u * n_imp, (size_t)n_imp, sizeof(int32_t), by_pos);
        if (n_tbm > 0) qsort(tbm_idx + u * n_tbm, (size_t)n_tbm, sizeof(int32_t), by_pos);
    }
    free(r);
    return REF_OK;
}

int ems_ref_select(const ems_ref_params* p, const double* s_glo, const double* s_loc,
                   double* s_pooled_opt, int32_t* imp_idx, int32_t* tbm_idx)
{
    if (!full_params_ok(p)) return REF_BAD;
    const size_t n = (size_t)p->batch * p->kv_heads * p->seq_len;
    double* s = s_pooled_opt ? s_pooled_opt : (double*)malloc(sizeof(double) * n);
    if (!s) return REF_BAD;
    int rc = ems_ref_combine_pool(p, s_glo, s_loc, s);
    if (rc == REF_OK) rc = ems_ref_partition(p, s, imp_idx, tbm_idx);
    if (!s_pooled_opt) free(s);
    return rc;
}

static double l2norm(const float* x, long D)
{
    double acc = 0.0;
    for (long d = 0; d < D; ++d) acc += (double)x[d] * (double)x[d];
    return sqrt(acc);
}

/* ------------------------------------------------------------------------------------
 * Eq. 5: d_i = argmax_d R[i][d] over the class centres, with R the cosine similarity of
 * the keys; tokens whose best similarity does not exceed tau go to the zero class
 * (Sec. 4.2).  A key of norm 0 has similarity 0 to everything.
 * ---------------------------------------------------------------------------------- */
int ems_ref_dest(const ems_ref_params* p, const float* k,
                 const int32_t* imp_idx, const int32_t* tbm_idx,
                 int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK || !k || !imp_idx) return REF_BAD;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest || !tbm_sim)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < BH; ++u) {
        const float* Ku = k + u * N * D;
        const int32_t* imp = imp_idx + u * n_imp;
        const int32_t* tbm = tbm_idx ? tbm_idx + u * n_tbm : NULL;
        double* cn = (double*)malloc(sizeof(double) * (size_t)n_imp);
        if (!cn) { bad = 1; continue; }
        for (long c = 0; c < n_imp; ++c) {
            cn[c] = l2norm(Ku + (long)imp[c] * D, D);
            if (k_norm_opt) k_norm_opt[u * (n_imp + n_tbm) + c] = cn[c];
        }
        for (long i = 0; i < n_tbm; ++i) {
            const float* ki = Ku + (long)tbm[i] * D;
            const double ni = l2norm(ki, D);
            if (k_norm_opt) k_norm_opt[u * (n_imp + n_tbm) + n_imp + i] = ni;
            double best = -INFINITY;
            int32_t arg = 0;
            for (long c = 0; c < n_imp; ++c) {
                const float* kc = Ku + (long)imp[c] * D;
                double sim = 0.0;
                if (ni > 0.0 && cn[c] > 0.0) {
                    for (long d = 0; d < D; ++d)
                        sim += ((double)ki[d] / ni) * ((double)kc[d] / cn[c]);
                }
                if (sim > best) { best = sim; arg = (int32_t)c; }
            }
            tbm_sim[u * n_tbm + i] = best;
            tbm_dest[u * n_tbm + i] = best > p->tau ? arg : p->budget;
        }
        free(cn);
    }
    return bad ? REF_BAD : REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Sec. 4.2 / App. A: N_tbm + N_imp tokens share N_imp entries, plus one zero-class
 * entry that collects the evicted ones.  Members of an entry = its centre and the TBM
 * tokens sent to it.  Values: arithmetic mean of the members.  Keys: only normalised
 * keys are merged and the norm is kept apart, so the entry's direction is the mean of
 * the members' unit keys and the stored row is that direction times the centre's own
 * norm.  The zero-class row keeps the plain means (scale 1).  An entry nobody joined
 * is the centre itself, copied.  Rows N_imp..budget-1 are the local tokens.
 * ---------------------------------------------------------------------------------- */
int ems_ref_merge(const ems_ref_params* p, const float* k, const float* v,
                  const int32_t* imp_idx, const int32_t* tbm_idx,
                  const int32_t* tbm_dest,
                  double* k_out, double* v_out, int32_t* kept_pos, int32_t* slot_count)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK) return REF_BAD;
    if (!k || !v || !imp_idx || !k_out || !v_out || !kept_pos || !slot_count) return REF_BAD;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
    const long Nb = p->budget, W = p->window, rows = Nb + 1;
    int bad = 0;
    for (long u = 0; u < BH; ++u) {
        for (long i = 0; i < n_tbm; ++i) {
            const int32_t d = tbm_dest[u * n_tbm + i];
            if (!((d >= 0 && d < n_imp) || d == Nb)) bad = 1;
        }
    }
    if (bad) return REF_BAD;

#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < BH; ++u) {
        const float* Ku = k + u * N * D;
        const float* Vu = v + u * N * D;
        const int32_t* imp = imp_idx + u * n_imp;
        const int32_t* tbm = tbm_idx ? tbm_idx + u * n_tbm : NULL;
        const int32_t* dst = tbm_dest ? tbm_dest + u * n_tbm : NULL;
        double* Ko = k_out + u * rows * D;
        double* Vo = v_out + u * rows * D;
        int32_t* cnt = slot_count + u * (n_imp + 1);
        int32_t* kp = kept_pos + u * Nb;

        for (long s = 0; s <= n_imp; ++s) {
            const int zero_class = (s == n_imp);
            const long row = zero_class ? Nb : s;
            double* ko = Ko + row * D;
            double* vo = Vo + row * D;
            for (long d = 0; d < D; ++d) { ko[d] = 0.0; vo[d] = 0.0; }
            long members = 0;
            double centre_norm = 1.0;
            if (!zero_class) {
                const float* kc = Ku + (long)imp[s] * D;
                const float* vc = Vu + (long)imp[s] * D;
                centre_norm = l2norm(kc, D);
                for (long d = 0; d < D; ++d) {
                    ko[d] += centre_norm > 0.0 ? (double)kc[d] / centre_norm : 0.0;
                    vo[d] += (double)vc[d];
                }
                members = 1;
            }
            for (long i = 0; i < n_tbm; ++i) {
                if (dst[i] != (zero_class ? Nb : s)) continue;
                const float* ki = Ku + (long)tbm[i] * D;
                const float* vi = Vu + (long)tbm[i] * D;
                const double ni = l2norm(ki, D);
                for (long d = 0; d < D; ++d) {
                    ko[d] += ni > 0.0 ? (double)ki[d] / ni : 0.0;
                    vo[d] += (double)vi[d];
                }
                ++members;
            }
            cnt[s] = (int32_t)members;
            if (!zero_class && members == 1) {
                const float* kc = Ku + (long)imp[s] * D;
                const float* vc = Vu + (long)imp[s] * D;
                for (long d = 0; d < D; ++d) { ko[d] = (double)kc[d]; vo[d] = (double)vc[d]; }
            } else if (members > 0) {
                for (long d = 0; d < D; ++d) {
                    ko[d] = centre_norm * (ko[d] / (double)members);
                    vo[d] = vo[d] / (double)members;
                }
            }
        }
        for (long s = 0; s < n_imp; ++s) kp[s] = imp[s];
        for (long t = 0; t < W; ++t) {
            const long pos = N - W + t;
            kp[n_imp + t] = (int32_t)pos;
            for (long d = 0; d < D; ++d) {
                Ko[(n_imp + t) * D + d] = (double)Ku[pos * D + d];
                Vo[(n_imp + t) * D + d] = (double)Vu[pos * D + d];
            }
        }
    }
    return REF_OK;
}

int ems_ref_evict_merge(const ems_ref_params* p, const float* k, const float* v,
                        const int32_t* imp_idx, const int32_t* tbm_idx,
                        double* k_out, double* v_out, int32_t* kept_pos,
                        int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt,
                        int32_t* slot_count)
{
    int rc = ems_ref_dest(p, k, imp_idx, tbm_idx, tbm_dest, tbm_sim, k_norm_opt);
    if (rc != REF_OK) return rc;
    return ems_ref_merge(p, k, v, imp_idx, tbm_idx, tbm_dest, k_out, v_out, kept_pos, slot_count);
}

/* ------------------------------------------------------------------------------------
 * Sec. 4.1 "Redundancy" and the similarity ablation of App. B: the redundancy R[i][d] that
 * Eq. 5 maximises is the key cosine, the value cosine, or -- the paper's own definition --
 * the product of the two.  similarity: 0 = key, 1 = value, 2 = key x value.  A vector of
 * norm 0 has cosine 0 to everything.  Threshold and tie-break as in ems_ref_dest; k_norm
 * always holds KEY norms.
 * ---------------------------------------------------------------------------------- */
static double cosine(const float* a, const float* b, long D)
{
    const double na = l2norm(a, D), nb = l2norm(b, D);
    if (!(na > 0.0) || !(nb > 0.0)) return 0.0;
    double dot = 0.0;
    for (long d = 0; d < D; ++d) dot += ((double)a[d] / na) * ((double)b[d] / nb);
    return dot;
}

int ems_ref_dest_sim(const ems_ref_params* p, int similarity, const float* k, const float* v,
                     const int32_t* imp_idx, const int32_t* tbm_idx,
                     int32_t* tbm_dest, double* tbm_sim, double* k_norm_opt)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK || !k || !v || !imp_idx) return REF_BAD;
    if (similarity < 0 || similarity > 2) return REF_BAD;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest || !tbm_sim)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < BH; ++u) {
        const float* Ku = k + u * N * D;
        const float* Vu = v + u * N * D;
        const int32_t* imp = imp_idx + u * n_imp;
        const int32_t* tbm = tbm_idx ? tbm_idx + u * n_tbm : NULL;
        if (k_norm_opt) {
            for (long c = 0; c < n_imp; ++c)
                k_norm_opt[u * (n_imp + n_tbm) + c] = l2norm(Ku + (long)imp[c] * D, D);
            for (long i = 0; i < n_tbm; ++i)
                k_norm_opt[u * (n_imp + n_tbm) + n_imp + i] = l2norm(Ku + (long)tbm[i] * D, D);
        }
        for (long i = 0; i < n_tbm; ++i) {
            double best = -INFINITY;
            int32_t arg = 0;
            for (long c = 0; c < n_imp; ++c) {
                const double ck = cosine(Ku + (long)tbm[i] * D, Ku + (long)imp[c] * D, D);
                const double cv = cosine(Vu + (long)tbm[i] * D, Vu + (long)imp[c] * D, D);
                const double r = similarity == 0 ? ck : similarity == 1 ? cv : ck * cv;
                if (r > best) { best = r; arg = (int32_t)c; }
            }
            tbm_sim[u * n_tbm + i] = best;
            tbm_dest[u * n_tbm + i] = best > p->tau ? arg : p->budget;
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Sec. 4.2, last paragraph: the merge is weighted by the tokens' attention scores so that
 * the more relevant members dominate.  `weight` is one non-negative score per token
 * ([B,Hkv,N]; negative entries count as 0).  With w_i the weight of member i of an entry
 * (centre included):
 *     value = sum w_i v_i / sum w_i ,   key = n_centre * sum w_i (k_i/|k_i|) / sum w_i .
 * An entry nobody joined, or whose weights add up to 0, stays the centre itself; a zero
 * class whose weights add up to 0 is a zero row.  slot_count still counts members.
 * ---------------------------------------------------------------------------------- */
int ems_ref_merge_weighted(const ems_ref_params* p, const float* k, const float* v,
                           const double* weight,
                           const int32_t* imp_idx, const int32_t* tbm_idx,
                           const int32_t* tbm_dest,
                           double* k_out, double* v_out, int32_t* kept_pos, int32_t* slot_count)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK) return REF_BAD;
    if (!k || !v || !weight || !imp_idx || !k_out || !v_out || !kept_pos || !slot_count) return REF_BAD;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
    const long Nb = p->budget, W = p->window, rows = Nb + 1;
    for (long u = 0; u < BH; ++u)
        for (long i = 0; i < n_tbm; ++i) {
            const int32_t d = tbm_dest[u * n_tbm + i];
            if (!((d >= 0 && d < n_imp) || d == Nb)) return REF_BAD;
        }

#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < BH; ++u) {
        const float* Ku = k + u * N * D;
        const float* Vu = v + u * N * D;
        const double* Wu = weight + u * N;
        const int32_t* imp = imp_idx + u * n_imp;
        const int32_t* tbm = tbm_idx ? tbm_idx + u * n_tbm : NULL;
        const int32_t* dst = tbm_dest ? tbm_dest + u * n_tbm : NULL;
        double* Ko = k_out + u * rows * D;
        double* Vo = v_out + u * rows * D;

        for (long s = 0; s <= n_imp; ++s) {
            const int zero_class = (s == n_imp);
            const long target = zero_class ? Nb : s;
            double* ko = Ko + target * D;
            double* vo = Vo + target * D;
            for (long d = 0; d < D; ++d) { ko[d] = 0.0; vo[d] = 0.0; }
            long members = 0;
            double total = 0.0, centre_norm = 1.0;
            /* member list: the centre first (if any), then the TBM tokens in order */
            for (long i = zero_class ? 0 : -1; i < n_tbm; ++i) {
                long pos;
                if (i < 0) pos = imp[s];
                else if (dst[i] == target) pos = tbm[i];
                else continue;
                const double ni = l2norm(Ku + pos * D, D);
                if (i < 0) centre_norm = ni;
                const double w = Wu[pos] > 0.0 ? Wu[pos] : 0.0;
                for (long d = 0; d < D; ++d) {
                    ko[d] += ni > 0.0 ? w * ((double)Ku[pos * D + d] / ni) : 0.0;
                    vo[d] += w * (double)Vu[pos * D + d];
                }
                total += w;
                ++members;
            }
            slot_count[u * (n_imp + 1) + s] = (int32_t)members;
            if (!zero_class && (members == 1 || !(total > 0.0))) {
                for (long d = 0; d < D; ++d) {
                    ko[d] = (double)Ku[(long)imp[s] * D + d];
                    vo[d] = (double)Vu[(long)imp[s] * D + d];
                }
            } else if (total > 0.0) {
                for (long d = 0; d < D; ++d) {
                    ko[d] = centre_norm * (ko[d] / total);
                    vo[d] = vo[d] / total;
                }
            } else {
                for (long d = 0; d < D; ++d) { ko[d] = 0.0; vo[d] = 0.0; }
            }
        }
        for (long s = 0; s < n_imp; ++s) kept_pos[u * Nb + s] = imp[s];
        for (long t = 0; t < W; ++t) {
            const long pos = N - W + t;
            kept_pos[u * Nb + n_imp + t] = (int32_t)pos;
            for (long d = 0; d < D; ++d) {
                Ko[(n_imp + t) * D + d] = (double)Ku[pos * D + d];
                Vo[(n_imp + t) * D + d] = (double)Vu[pos * D + d];
            }
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Eq. 3: sparsity rate of a head.  s = Eq. 2 score (no pooling) sorted in descending
 * order; N_k = the smallest count whose leading scores add up to at least zeta of the
 * total; p = 1 - N_k / N.  (The equation prints the bare threshold zeta; the sentence
 * before it says "over zeta of the total score", so the scores are taken relative to
 * their sum.)  p_out [B,Hkv]; n_k_opt [B,Hkv] nullable.
 * ---------------------------------------------------------------------------------- */
static int desc_double(const void* a, const void* b)
{
    const double x = *(const double*)a, y = *(const double*)b;
    return (x < y) - (x > y);
}

int ems_ref_sparsity(const ems_ref_params* p, double zeta, const double* s_glo, const double* s_loc,
                     double* p_out, int32_t* n_k_opt)
{
    if (!score_params_ok(p) || !s_glo || !s_loc || !p_out) return REF_BAD;
    if (!(zeta > 0.0) || !(zeta <= 1.0)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len;
    double* s = (double*)malloc(sizeof(double) * (size_t)N);
    if (!s) return REF_BAD;
    for (long u = 0; u < BH; ++u) {
        const double* g = s_glo + u * N;
        const double* l = s_loc + u * N;
        double sg = 0.0, sl = 0.0;
        for (long j = 0; j < N; ++j) { sg += g[j]; sl += l[j]; }
        const double c = sg > 0.0 ? (sl / (double)N) / (sg / (double)N) : 0.0;      /* Eq. 2 */
        double total = 0.0;
        for (long j = 0; j < N; ++j) { s[j] = fmax(g[j] * c, l[j]); total += s[j]; }
        qsort(s, (size_t)N, sizeof(double), desc_double);
        double run = 0.0;
        long nk = N;
        for (long i = 0; i < N; ++i) {
            run += s[i];
            if (run >= zeta * total) { nk = i + 1; break; }
        }
        p_out[u] = 1.0 - (double)nk / (double)N;
        if (n_k_opt) n_k_opt[u] = (int32_t)nk;
    }
    free(s);
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Eq. 4: redundancy rate of a head.  R[k][j] = cos(key_k, key_j) * cos(value_k, value_j)
 * (Sec. 4.1); token k is redundant if some EARLIER token j < k ("another token in the
 * existing KV cache") has R[k][j] >= tau; r = (number of redundant tokens) / N.  The first
 * token has no predecessor.  r_out [B,Hkv]; best_opt [B,Hkv,N] = max_j<k R[k][j] (-inf for
 * k = 0), nullable.
 * ---------------------------------------------------------------------------------- */
int ems_ref_redundancy(const ems_ref_params* p, const float* k, const float* v,
                       double* r_out, double* best_opt)
{
    if (!score_params_ok(p) || !k || !v || !r_out) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
    for (long u = 0; u < BH; ++u) {
        const float* Ku = k + u * N * D;
        const float* Vu = v + u * N * D;
        long redundant = 0;
#pragma omp parallel for schedule(dynamic, 8) reduction(+ : redundant)
        for (long t = 0; t < N; ++t) {
            double best = -INFINITY;
            for (long j = 0; j < t; ++j) {
                const double r = cosine(Ku + t * D, Ku + j * D, D) * cosine(Vu + t * D, Vu + j * D, D);
                if (r > best) best = r;
            }
            if (best_opt) best_opt[u * N + t] = best;
            if (best >= p->tau) ++redundant;
        }
        r_out[u] = (double)redundant / (double)N;
    }
    return REF_OK;
}

/* Eq. 4's inner maximum for chosen tokens only (the same loop as ems_ref_redundancy, for
 * sequences where all N^2/2 pairs are too many): best_out[u][i] = max_j<t R[t][j] with
 * t = tokens[i], for every (batch, kv-head) unit u.  best_out [B,Hkv,n_tokens]. */
int ems_ref_redundancy_at(const ems_ref_params* p, const float* k, const float* v,
                          const int32_t* tokens, int32_t n_tokens, double* best_out)
{
    if (!score_params_ok(p) || !k || !v || !tokens || n_tokens < 0 || !best_out) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, N = p->seq_len, D = p->head_dim;
    for (long i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= N) return REF_BAD;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long u = 0; u < BH; ++u) {
        for (long i = 0; i < n_tokens; ++i) {
            const float* Ku = k + u * N * D;
            const float* Vu = v + u * N * D;
            const long t = tokens[i];
            double best = -INFINITY;
            for (long j = 0; j < t; ++j) {
                const double r = cosine(Ku + t * D, Ku + j * D, D) * cosine(Vu + t * D, Vu + j * D, D);
                if (r > best) best = r;
            }
            best_out[u * n_tokens + i] = best;
        }
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------------------
 * App. A, "Shared Entry Expansion": tokens that were merged share one cache entry; at
 * compute time the entry is expanded back to one key/value per token with the help of
 * the look-up-table (which entry each token went to) and the stored key norms (Sec. 4.2:
 * only normalised keys are merged, the norm is kept as one scalar per token).
 * ---------------------------------------------------------------------------------- */
int ems_ref_expand(const ems_ref_params* p, const double* k_cache, const double* v_cache,
                   const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
                   const double* k_norm, double* k_exp, double* v_exp, int32_t* pos_exp)
{
    int32_t n_imp, n_tbm;
    if (ems_ref_sizes(p, &n_imp, &n_tbm) != REF_OK) return REF_BAD;
    if (!k_cache || !v_cache || !kept_pos || !k_norm || !k_exp || !v_exp || !pos_exp) return REF_BAD;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest)) return REF_BAD;
    const long BH = (long)p->batch * p->kv_heads, D = p->head_dim;
    const long Nb = p->budget, W = p->window, E = n_imp + n_tbm + W;
    for (long u = 0; u < BH; ++u) {
        const double* Kc = k_cache + u * (Nb + 1) * D;
        const double* Vc = v_cache + u * (Nb + 1) * D;
        const double* nrm = k_norm + u * (n_imp + n_tbm);
        double* Ke = k_exp + u * E * D;
        double* Ve = v_exp + u * E * D;
        int32_t* pe = pos_exp + u * E;
        for (long s = 0; s < n_imp; ++s) {                  /* a centre is its entry */
            for (long d = 0; d < D; ++d) { Ke[s * D + d] = Kc[s * D + d]; Ve[s * D + d] = Vc[s * D + d]; }
            pe[s] = kept_pos[u * Nb + s];
        }
        for (long i = 0; i < n_tbm; ++i) {
            const long row = n_imp + i;
            const int32_t s = tbm_dest[u * n_tbm + i];
            if (s >= 0 && s < n_imp) {
                const double nc = nrm[s], ni = nrm[n_imp + i];
                for (long d = 0; d < D; ++d) {
                    const double dir = nc > 0.0 ? Kc[s * D + d] / nc : 0.0;   /* entry direction */
                    Ke[row * D + d] = ni * dir;
                    Ve[row * D + d] = Vc[s * D + d];
                }
                pe[row] = tbm_idx[u * n_tbm + i];
            } else if (s == Nb) {                           /* zero class: evicted */
                for (long d = 0; d < D; ++d) { Ke[row * D + d] = 0.0; Ve[row * D + d] = 0.0; }
                pe[row] = -1;
            } else {
                return REF_BAD;
            }
        }
        for (long t = 0; t < W; ++t) {                      /* local tokens are their own entries */
            const long row = n_imp + n_tbm + t, src = n_imp + t;
            for (long d = 0; d < D; ++d) { Ke[row * D + d] = Kc[src * D + d]; Ve[row * D + d] = Vc[src * D + d]; }
            pe[row] = kept_pos[u * Nb + src];
        }
    }
    return REF_OK;
}
