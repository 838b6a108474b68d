// Host side of the C ABI declared in include/ems.h: argument validation, workspace
// carving and kernel launches.  Nothing here allocates, frees or synchronises.
#include "../../include/ems.h"
#include "ems_kernels.h"

#include <cmath>
#include <mutex>

namespace {

// Scratch of ems_evict_merge_static: a fixed array in every device's global memory, part of
// the loaded code object, so nothing is allocated for it at run time.  In host code the
// array's name is only a handle; its address on a device comes from hipGetSymbolAddress,
// asked once per device (static_scratch below) and kept.
constexpr size_t kStaticScratchBytes = EMS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch`, or nullptr with *err set.
void* static_scratch(hipError_t* err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool score_params_ok(const ems_params* p, int* why)
{
    *why = EMS_ERR_INVALID_ARG;
    if (!p) return false;
    if (p->batch < 1 || p->q_heads < 1 || p->kv_heads < 1) return false;
    if (p->q_heads % p->kv_heads) return false;
    if (p->seq_len < 1 || p->window < 1 || p->window > p->seq_len) return false;
    if (p->dtype != EMS_BF16 && p->dtype != EMS_F32) return false;
    if (p->head_dim < 1) return false;
    if (std::isnan(p->softmax_scale) || std::isinf(p->softmax_scale)) return false;
    *why = EMS_ERR_UNSUPPORTED;
    if (p->head_dim != 64 && p->head_dim != 128) return false;
    if (p->seq_len > (1 << 22)) return false;                       // 32-bit index headroom
    if ((long long)p->batch * p->kv_heads > 65535) return false;    // grid.y
    if ((long long)p->batch * p->q_heads * ((p->seq_len + 127) / 128) > (1ll << 30)) return false;
    return true;
}

bool full_params_ok(const ems_params* p, int* why)
{
    if (!score_params_ok(p, why)) return false;
    *why = EMS_ERR_INVALID_ARG;
    if (!(p->window < p->budget && p->budget <= p->seq_len)) return false;
    if (p->pool_kernel < 1 || p->pool_kernel > 63 || (p->pool_kernel % 2) == 0) return false;
    if (!(p->merge_ratio >= 0.f) || std::isinf(p->merge_ratio)) return false;
    if (std::isnan(p->tau)) return false;
    return true;
}

void partition_sizes(const ems_params* p, int* n_imp, int* n_tbm)
{
    // Sec. 4.2: N_budget = N_imp + L_win, gamma = (N_budget + N_tbm) / N_budget = 1 + r
    *n_imp = p->budget - p->window;
    const double want = std::floor((double)p->merge_ratio * (double)p->budget);
    const int room = p->seq_len - p->budget;
    *n_tbm = want > (double)room ? room : (int)want;
}

struct ScorePlan {
    int n_chunks, chunk_rows, loc_chunk0, n_pad, p1_splits;
    size_t off_lse2, off_part_glo, off_part_loc, off_part_m, off_part_l, off_queue, total;
};

// Row chunks of the key-stationary pass: small enough that there are tens of thousands of
// (key tile, row chunk) work items -- one wave each, 1024 waves resident -- so that the last
// items to finish are a small part of the run, large enough that the keys a wave holds in
// registers are reused over many rows.
ScorePlan plan_score(const ems_params* p)
{
    ScorePlan s{};
    const int N = p->seq_len;
    const long long bkv = (long long)p->batch * p->kv_heads;
    const int kpb = ems::score_keys_per_block(p->dtype == EMS_F32);
    const int n_key_tiles = (N + kpb - 1) / kpb;
    auto items = [&](int R) {
        const int nI = (N + R - 1) / R;
        long long t = 0;
        for (int J = 0; J < n_key_tiles; ++J) t += nI - (int)(((long long)J * kpb) / R);
        return t * bkv;
    };
    int R = 4096;
    while (R > 512 && items(R) < 32768) R >>= 1;
    s.chunk_rows = R;
    s.n_chunks = (N + R - 1) / R;
    s.loc_chunk0 = (N - p->window) / R;
    size_t off = 0;
    s.n_pad = (N + 63) / 64 * 64;
    s.off_lse2 = off; off += align_up(sizeof(float) * (size_t)p->batch * p->q_heads * s.n_pad);
    s.off_part_glo = off;
    s.off_part_loc = off;
    if (s.n_chunks > 1) {
        off += align_up(sizeof(float) * (size_t)bkv * s.n_chunks * N);
        s.off_part_loc = off;
        off += align_up(sizeof(float) * (size_t)bkv * (s.n_chunks - s.loc_chunk0) * N);
    }
    // Pass 1: a row tile's key range is cut into splits while there are too few row tiles to
    // balance the causal triangle over the chip (short sequences); partial (max, sum) pairs
    // are then combined by a small kernel.
    const int rpb = kpb;                                              // query rows per pass-1 wave
    const long long row_tiles = (long long)p->batch * p->q_heads * ((N + rpb - 1) / rpb);
    s.p1_splits = 1;
    while (s.p1_splits < 8 && row_tiles * s.p1_splits < 2048 && (N + rpb - 1) / rpb >= 2 * s.p1_splits) s.p1_splits *= 2;
    s.off_part_m = off; s.off_part_l = off;
    if (s.p1_splits > 1) {
        const size_t one = align_up(sizeof(float) * (size_t)s.p1_splits * p->batch * p->q_heads * s.n_pad);
        off += one; s.off_part_l = off; off += one;
    }
    s.off_queue = off; off += kAlign;                                   // work-queue cursors of the second pass
    s.total = off;
    return s;
}

struct SelectPlan { size_t off_pooled, off_ckey, off_cpos, off_hist, off_sums, off_count, off_info, total; };

SelectPlan plan_select(const ems_params* p)
{
    SelectPlan s{};
    const size_t bkv = (size_t)p->batch * p->kv_heads, N = (size_t)p->seq_len;
    const size_t chunks = (size_t)ems::select_chunks(p->seq_len);
    size_t off = 0;
    s.off_pooled = off; off += align_up(sizeof(float) * bkv * N);       // ranking keys
    s.off_ckey = off; off += align_up(sizeof(uint32_t) * bkv * N);      // candidate list (long sequences)
    s.off_cpos = off; off += align_up(sizeof(int32_t) * bkv * N);
    s.off_hist = off; off += align_up(sizeof(int) * bkv * (size_t)ems::select_coarse_bins());
    s.off_sums = off; off += align_up(sizeof(float) * bkv * chunks * 2);
    s.off_count = off; off += align_up(sizeof(int) * bkv * chunks * 2);
    s.off_info = off; off += align_up(sizeof(int) * bkv * 2);
    s.total = off;
    return s;
}

size_t select_ws_bytes(const ems_params* p) { return plan_select(p).total; }

// Evict-merge workspace: the key norms (used when the caller does not ask for them) and, when the
// centre list is searched in slices, the per-slice winners.
struct MergePlan {
    int slice_rows, n_slices;
    size_t off_norm, off_best, off_arg, total;
};

MergePlan plan_merge(const ems_params* p)
{
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    MergePlan m{};
    ems::dest_slicing(n_imp, p->dtype == EMS_F32, &m.slice_rows, &m.n_slices);
    const size_t bkv = (size_t)p->batch * p->kv_heads;
    const size_t part = m.n_slices > 1 ? align_up(4 * bkv * m.n_slices * (size_t)n_tbm) : 0;
    m.off_norm = 0;
    m.off_best = align_up(sizeof(float) * bkv * (size_t)(n_imp + n_tbm));
    m.off_arg = m.off_best + part;
    m.total = m.off_arg + part;
    return m;
}

size_t merge_ws_bytes(const ems_params* p) { return plan_merge(p).total; }

bool ws_ok(const void* ws, size_t have, size_t need)
{
    return ws && ((uintptr_t)ws % kAlign) == 0 && have >= need;
}

}  // namespace

extern "C" {

int ems_version(void) { return 200; }

const char* ems_strerror(int status)
{
    switch (status) {
        case EMS_OK: return "ok";
        case EMS_ERR_INVALID_ARG: return "invalid argument";
        case EMS_ERR_UNSUPPORTED: return "unsupported configuration";
        case EMS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case EMS_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int ems_partition_sizes(const ems_params* p, int32_t* n_imp, int32_t* n_tbm)
{
    int why;
    if (!full_params_ok(p, &why)) return why;
    int a, b;
    partition_sizes(p, &a, &b);
    if (n_imp) *n_imp = a;
    if (n_tbm) *n_tbm = b;
    return EMS_OK;
}

int ems_workspace_bytes(const ems_params* p, size_t* score_ws, size_t* select_ws, size_t* merge_ws)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (score_ws) *score_ws = plan_score(p).total;
    if (select_ws || merge_ws) {
        if (!full_params_ok(p, &why)) return why;
        if (select_ws) *select_ws = select_ws_bytes(p);
        if (merge_ws) *merge_ws = merge_ws_bytes(p);
    }
    return EMS_OK;
}

static void fill_score_args(ems::ScoreArgs& a, const ems_params* p, const ScorePlan& plan, void* ws)
{
    char* w = static_cast<char*>(ws);
    a.lse2 = w ? reinterpret_cast<float*>(w + plan.off_lse2) : nullptr;
    a.part_glo = w ? reinterpret_cast<float*>(w + plan.off_part_glo) : nullptr;
    a.part_loc = w ? reinterpret_cast<float*>(w + plan.off_part_loc) : nullptr;
    a.part_m = w ? reinterpret_cast<float*>(w + plan.off_part_m) : nullptr;
    a.part_l = w ? reinterpret_cast<float*>(w + plan.off_part_l) : nullptr;
    a.queue = w ? reinterpret_cast<int*>(w + plan.off_queue) : nullptr;
    a.p1_splits = plan.p1_splits;
    a.batch = p->batch; a.q_heads = p->q_heads; a.kv_heads = p->kv_heads;
    a.head_dim = p->head_dim; a.seq_len = p->seq_len; a.window = p->window;
    a.n_pad = plan.n_pad;
    a.n_chunks = plan.n_chunks; a.chunk_rows = plan.chunk_rows; a.loc_chunk0 = plan.loc_chunk0;
    const double scale = p->softmax_scale > 0.f ? (double)p->softmax_scale
                                                : 1.0 / std::sqrt((double)p->head_dim);   // Eq. 1
    a.scale_log2e = (float)(scale * 1.4426950408889634074);
}

int ems_global_local_score(const ems_params* p, const void* q, const void* k,
                           float* s_glo, float* s_loc, float* lse_opt,
                           void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (!q || !k || !s_glo || !s_loc) return EMS_ERR_INVALID_ARG;
    const ScorePlan plan = plan_score(p);
    if (!ws_ok(ws, ws_bytes, plan.total)) return EMS_ERR_WORKSPACE;

    ems::ScoreArgs a{};
    a.q = q; a.k = k; a.s_glo = s_glo; a.s_loc = s_loc; a.lse_opt = lse_opt;
    fill_score_args(a, p, plan, ws);
    const hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = ems::launch_score_pass1(a, p->dtype == EMS_F32, st);
    if (e == hipSuccess) e = ems::launch_score_pass2(a, p->dtype == EMS_F32, st);
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_attention_lse(const ems_params* p, const void* q, const void* k, float* lse,
                      void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (!q || !k || !lse) return EMS_ERR_INVALID_ARG;
    const ScorePlan plan = plan_score(p);
    if (!ws_ok(ws, ws_bytes, plan.total)) return EMS_ERR_WORKSPACE;
    ems::ScoreArgs a{};
    a.q = q; a.k = k; a.lse_opt = lse;
    fill_score_args(a, p, plan, ws);
    const hipError_t e = ems::launch_score_pass1(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_global_local_score_from_lse(const ems_params* p, const void* q, const void* k,
                                    const float* lse, float* s_glo, float* s_loc,
                                    void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (!q || !k || !lse || !s_glo || !s_loc) return EMS_ERR_INVALID_ARG;
    const ScorePlan plan = plan_score(p);
    if (!ws_ok(ws, ws_bytes, plan.total)) return EMS_ERR_WORKSPACE;
    ems::ScoreArgs a{};
    a.q = q; a.k = k; a.s_glo = s_glo; a.s_loc = s_loc; a.lse_in_nat = lse;
    fill_score_args(a, p, plan, ws);
    const hipError_t e = ems::launch_score_pass2(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_select(const ems_params* p, const float* s_glo, const float* s_loc,
               float* s_gl_opt, int32_t* imp_idx, int32_t* tbm_idx,
               void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!full_params_ok(p, &why)) return why;
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    if (!s_glo || !s_loc || !imp_idx || (n_tbm > 0 && !tbm_idx)) return EMS_ERR_INVALID_ARG;
    if (!ws_ok(ws, ws_bytes, select_ws_bytes(p))) return EMS_ERR_WORKSPACE;

    ems::SelectArgs a{};
    a.s_glo = s_glo; a.s_loc = s_loc; a.s_gl_opt = s_gl_opt;
    const SelectPlan sp = plan_select(p);
    char* w = static_cast<char*>(ws);
    a.pooled = reinterpret_cast<float*>(w + sp.off_pooled);
    a.cand_key = reinterpret_cast<uint32_t*>(w + sp.off_ckey);
    a.cand_pos = reinterpret_cast<int32_t*>(w + sp.off_cpos);
    a.coarse_hist = reinterpret_cast<int*>(w + sp.off_hist);
    a.chunk_sums = reinterpret_cast<float*>(w + sp.off_sums);
    a.chunk_count = reinterpret_cast<int*>(w + sp.off_count);
    a.head_info = reinterpret_cast<int*>(w + sp.off_info);
    a.n_chunks = ems::select_chunks(p->seq_len);
    a.imp_idx = imp_idx; a.tbm_idx = tbm_idx;
    a.bkv = p->batch * p->kv_heads; a.seq_len = p->seq_len; a.window = p->window;
    a.n_imp = n_imp; a.n_tbm = n_tbm; a.pool_kernel = p->pool_kernel;
    const hipError_t e = ems::launch_select(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

// Argument checks shared by the evict-merge entry points.
static bool evict_merge_args_ok(const ems_params* p, int similarity, const void* k, const void* v,
                                const int32_t* imp_idx, const int32_t* tbm_idx,
                                const void* k_out, const void* v_out, const int32_t* kept_pos,
                                const int32_t* tbm_dest, const float* tbm_sim, const int32_t* slot_count,
                                int* why)
{
    if (!full_params_ok(p, why)) return false;
    *why = EMS_ERR_INVALID_ARG;
    if (similarity != EMS_SIM_KEY && similarity != EMS_SIM_VALUE && similarity != EMS_SIM_KEY_VALUE) return false;
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    if (!k || !v || !imp_idx || !k_out || !v_out || !kept_pos || !slot_count) return false;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest || !tbm_sim)) return false;
    return true;
}

// Kernel launches of the evict-merge stage on checked arguments; `ws` holds merge_ws_bytes(p).
static int evict_merge_launch(const ems_params* p, int similarity, const void* k, const void* v,
                              const float* token_weight_opt,
                              const int32_t* imp_idx, const int32_t* tbm_idx,
                              void* k_out, void* v_out, int32_t* kept_pos,
                              int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                              int32_t* slot_count, void* ws, void* hip_stream)
{
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);

    ems::MergeArgs a{};
    a.k = k; a.v = v; a.imp_idx = imp_idx; a.tbm_idx = tbm_idx;
    a.k_out = k_out; a.v_out = v_out; a.kept_pos = kept_pos;
    a.tbm_dest = tbm_dest; a.tbm_sim = tbm_sim;
    const MergePlan plan = plan_merge(p);
    char* w = static_cast<char*>(ws);
    a.k_norm = k_norm_opt ? k_norm_opt : reinterpret_cast<float*>(w + plan.off_norm);
    a.slice_rows = plan.slice_rows; a.n_slices = plan.n_slices;
    a.part_best = reinterpret_cast<float*>(w + plan.off_best);
    a.part_arg = reinterpret_cast<int32_t*>(w + plan.off_arg);
    a.slot_count = slot_count;
    a.bkv = p->batch * p->kv_heads; a.head_dim = p->head_dim; a.seq_len = p->seq_len;
    a.window = p->window; a.budget = p->budget; a.n_imp = n_imp; a.n_tbm = n_tbm;
    a.tau = p->tau;
    a.weight = token_weight_opt; a.similarity = similarity;
    const hipError_t e = ems::launch_evict_merge(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_evict_merge(const ems_params* p, const void* k, const void* v,
                    const int32_t* imp_idx, const int32_t* tbm_idx,
                    void* k_out, void* v_out, int32_t* kept_pos,
                    int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                    int32_t* slot_count,
                    void* ws, size_t ws_bytes, void* hip_stream)
{
    return ems_evict_merge_variant(p, EMS_SIM_KEY, k, v, nullptr, imp_idx, tbm_idx, k_out, v_out, kept_pos,
                                   tbm_dest, tbm_sim, k_norm_opt, slot_count, ws, ws_bytes, hip_stream);
}

int ems_evict_merge_variant(const ems_params* p, int similarity, const void* k, const void* v,
                            const float* token_weight_opt,
                            const int32_t* imp_idx, const int32_t* tbm_idx,
                            void* k_out, void* v_out, int32_t* kept_pos,
                            int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                            int32_t* slot_count,
                            void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!evict_merge_args_ok(p, similarity, k, v, imp_idx, tbm_idx, k_out, v_out, kept_pos,
                             tbm_dest, tbm_sim, slot_count, &why)) return why;
    if (!ws_ok(ws, ws_bytes, merge_ws_bytes(p))) return EMS_ERR_WORKSPACE;
    return evict_merge_launch(p, similarity, k, v, token_weight_opt, imp_idx, tbm_idx, k_out, v_out, kept_pos,
                              tbm_dest, tbm_sim, k_norm_opt, slot_count, ws, hip_stream);
}

int ems_evict_merge_static(const ems_params* p, const void* k, const void* v,
                           const int32_t* imp_idx, const int32_t* tbm_idx,
                           void* k_out, void* v_out, int32_t* kept_pos,
                           int32_t* tbm_dest, float* tbm_sim, float* k_norm_opt,
                           int32_t* slot_count, void* hip_stream)
{
    int why;
    if (!evict_merge_args_ok(p, EMS_SIM_KEY, k, v, imp_idx, tbm_idx, k_out, v_out, kept_pos,
                             tbm_dest, tbm_sim, slot_count, &why)) return why;
    if (merge_ws_bytes(p) > kStaticScratchBytes) return EMS_ERR_WORKSPACE;
    hipError_t err;
    void* ws = static_scratch(&err);
    if (!ws) return EMS_ERR_LAUNCH;
    return evict_merge_launch(p, EMS_SIM_KEY, k, v, nullptr, imp_idx, tbm_idx, k_out, v_out, kept_pos,
                              tbm_dest, tbm_sim, k_norm_opt, slot_count, ws, hip_stream);
}

int ems_expand(const ems_params* p, const void* k_cache, const void* v_cache,
               const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
               const float* k_norm, void* k_exp, void* v_exp, int32_t* pos_exp,
               void* hip_stream)
{
    int why;
    if (!full_params_ok(p, &why)) return why;
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    if (!k_cache || !v_cache || !kept_pos || !k_norm || !k_exp || !v_exp || !pos_exp) return EMS_ERR_INVALID_ARG;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest)) return EMS_ERR_INVALID_ARG;
    ems::ExpandArgs a{};
    a.k_cache = k_cache; a.v_cache = v_cache; a.kept_pos = kept_pos; a.tbm_idx = tbm_idx;
    a.tbm_dest = tbm_dest; a.k_norm = k_norm; a.k_exp = k_exp; a.v_exp = v_exp; a.pos_exp = pos_exp;
    a.bkv = p->batch * p->kv_heads; a.head_dim = p->head_dim; a.window = p->window;
    a.budget = p->budget; a.n_imp = n_imp; a.n_tbm = n_tbm;
    const hipError_t e = ems::launch_expand(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_sparsity_rate(const ems_params* p, float zeta, const float* s_glo, const float* s_loc,
                      float* rate, int32_t* n_k_opt, void* hip_stream)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (!s_glo || !s_loc || !rate || !(zeta > 0.f) || !(zeta <= 1.f)) return EMS_ERR_INVALID_ARG;
    ems::StatsArgs a{};
    a.s_glo = s_glo; a.s_loc = s_loc; a.p_out = rate; a.n_k_opt = n_k_opt;
    a.bkv = p->batch * p->kv_heads; a.head_dim = p->head_dim; a.seq_len = p->seq_len; a.zeta = zeta;
    const hipError_t e = ems::launch_sparsity(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_redundancy_rate(const ems_params* p, const void* k, const void* v,
                        float* rate, float* best, void* hip_stream)
{
    int why;
    if (!score_params_ok(p, &why)) return why;
    if (!k || !v || !rate || !best || std::isnan(p->tau)) return EMS_ERR_INVALID_ARG;
    ems::StatsArgs a{};
    a.k = k; a.v = v; a.r_out = rate; a.best = best;
    a.bkv = p->batch * p->kv_heads; a.head_dim = p->head_dim; a.seq_len = p->seq_len; a.tau = p->tau;
    const hipError_t e = ems::launch_redundancy(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

static bool decode_params_ok(const ems_params* p, int* why)
{
    if (!full_params_ok(p, why)) return false;
    const int g = p->q_heads / p->kv_heads;
    *why = EMS_ERR_UNSUPPORTED;
    return g == 1 || g == 2 || g == 4 || g == 8;
}

// Decode-step workspace: the staged row dots and row norms, then (large caches) the hand-over
// records of the sliced step.
static size_t decode_stage_bytes(const ems_params* p)
{
    const size_t bkv = (size_t)p->batch * p->kv_heads;
    const size_t g = (size_t)(p->q_heads / p->kv_heads);
    return align_up(sizeof(float) * bkv * (g + 1) * (size_t)p->budget);
}

static size_t decode_ws_bytes(const ems_params* p)
{
    int n_imp, n_tbm, slice_rows, n_slices;
    partition_sizes(p, &n_imp, &n_tbm);
    const bool split = ems::decode_split(p->budget, n_imp, n_tbm, p->window, p->dtype == EMS_F32, &slice_rows, &n_slices);
    const size_t bkv = (size_t)p->batch * p->kv_heads;
    return decode_stage_bytes(p) + (split ? align_up(sizeof(float) * bkv * ems::kDecodeHandFloats) : 0);
}

static bool state_ok(const ems_decode_state* s)
{
    return s && s->k_cache && s->v_cache && s->row_norm && s->entry_count && s->entry_tok && s->tok_pos &&
           s->tok_row && s->tok_norm && s->tok_glo && s->tok_past && s->tok_cur && s->step_count;
}

static ems::DecodeState to_internal(const ems_decode_state* s)
{
    ems::DecodeState d{};
    d.k_cache = s->k_cache; d.v_cache = s->v_cache; d.row_norm = s->row_norm;
    d.entry_count = s->entry_count; d.entry_tok = s->entry_tok; d.tok_pos = s->tok_pos;
    d.tok_row = s->tok_row; d.tok_norm = s->tok_norm; d.tok_glo = s->tok_glo;
    d.tok_past = s->tok_past; d.tok_cur = s->tok_cur; d.step_count = s->step_count;
    return d;
}

int ems_decode_workspace_bytes(const ems_params* p, size_t* decode_ws)
{
    int why;
    if (!decode_params_ok(p, &why)) return why;
    if (decode_ws) *decode_ws = decode_ws_bytes(p);
    return EMS_OK;
}

int ems_decode_init(const ems_params* p, const float* s_glo, const float* s_loc,
                    const int32_t* kept_pos, const int32_t* tbm_idx, const int32_t* tbm_dest,
                    const float* k_norm, const int32_t* slot_count,
                    const ems_decode_state* state, void* hip_stream)
{
    int why;
    if (!decode_params_ok(p, &why)) return why;
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    if (!s_glo || !s_loc || !kept_pos || !k_norm || !slot_count || !state_ok(state)) return EMS_ERR_INVALID_ARG;
    if (n_tbm > 0 && (!tbm_idx || !tbm_dest)) return EMS_ERR_INVALID_ARG;
    ems::DecodeInitArgs a{};
    a.st = to_internal(state);
    a.s_glo = s_glo; a.s_loc = s_loc; a.kept_pos = kept_pos; a.tbm_idx = tbm_idx; a.tbm_dest = tbm_dest;
    a.k_norm = k_norm; a.slot_count = slot_count;
    a.bkv = p->batch * p->kv_heads; a.head_dim = p->head_dim; a.seq_len = p->seq_len;
    a.window = p->window; a.budget = p->budget; a.n_imp = n_imp; a.n_tbm = n_tbm;
    const hipError_t e = ems::launch_decode_init(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

int ems_decode_step(const ems_params* p, const ems_decode_state* state, int32_t step,
                    const void* q_new, const void* k_new, const void* v_new,
                    float* attn_opt, int32_t* decision_opt, float* sim_opt,
                    void* ws, size_t ws_bytes, void* hip_stream)
{
    int why;
    if (!decode_params_ok(p, &why)) return why;
    int n_imp, n_tbm;
    partition_sizes(p, &n_imp, &n_tbm);
    if (!state_ok(state) || !q_new || !k_new || !v_new) return EMS_ERR_INVALID_ARG;
    if (step < EMS_STEP_FROM_STATE || (long long)p->seq_len + step > 0x7fffffffll) return EMS_ERR_INVALID_ARG;
    if (!ws_ok(ws, ws_bytes, decode_ws_bytes(p))) return EMS_ERR_WORKSPACE;
    const size_t bkv = (size_t)p->batch * p->kv_heads;
    const int g = p->q_heads / p->kv_heads;
    ems::DecodeStepArgs a{};
    a.st = to_internal(state);
    a.q_new = q_new; a.k_new = k_new; a.v_new = v_new;
    a.attn_opt = attn_opt; a.decision_opt = decision_opt; a.sim_opt = sim_opt;
    a.ws = static_cast<float*>(ws);
    if (ems::decode_split(p->budget, n_imp, n_tbm, p->window, p->dtype == EMS_F32, &a.slice_rows, &a.n_slices))
        a.hand = reinterpret_cast<float*>(static_cast<char*>(ws) + decode_stage_bytes(p));
    // per-row dot products and row norms are staged in LDS when they fit in
    // what a block may ask for without raising the limit, else in the workspace
    const size_t stage_floats = (size_t)(g + 1) * p->budget;
    a.lds_floats = stage_floats * sizeof(float) <= 60 * 1024 ? (int)stage_floats : 0;
    a.bkv = (int)bkv; a.group = g; a.head_dim = p->head_dim; a.window = p->window; a.budget = p->budget;
    a.n_imp = n_imp; a.n_tbm = n_tbm; a.step = step; a.seq_len = p->seq_len;
    a.tau = p->tau;
    const double scale = p->softmax_scale > 0.f ? (double)p->softmax_scale : 1.0 / std::sqrt((double)p->head_dim);
    a.scale_log2e = (float)(scale * 1.4426950408889634074);
    const hipError_t e = ems::launch_decode_step(a, p->dtype == EMS_F32, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? EMS_OK : EMS_ERR_LAUNCH;
}

}  // extern "C"
