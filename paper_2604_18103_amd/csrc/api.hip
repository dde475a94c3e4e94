// Host side of libdash: argument validation, workspace carving, stage sequencing. See include/dash.h.
#include <math.h>
#include <new>

#include "common.h"

using namespace dash;

struct dash_profile {
    hipEvent_t ev[DASH_N_STAGES + 1];
    bool recorded;
    bool merged;  // stages 2 and 3 ran as one launch: ev[3] was not recorded
};

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t elem_size(int dtype) { return dtype == DASH_BF16 ? 2 : 4; }

dash_status check_params(const dash_layer_params* p) {
    if (!p) return DASH_ERR_INVALID_ARG;
    if (p->dtype != DASH_BF16 && p->dtype != DASH_F32) return DASH_ERR_INVALID_ARG;
    if (p->d <= 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0) return DASH_ERR_INVALID_ARG;
    if (p->n_q_heads % p->n_kv_heads != 0) return DASH_ERR_INVALID_ARG;
    if (p->head_dim != 64 && p->head_dim != 128) return DASH_ERR_UNSUPPORTED;
    if ((p->d * (int)elem_size(p->dtype)) % 16 != 0) return DASH_ERR_UNSUPPORTED;  // 16-byte row vectors
    if (p->rule != DASH_RULE_NONE && p->rule != DASH_RULE_THRESHOLD && p->rule != DASH_RULE_TOPK)
        return DASH_ERR_INVALID_ARG;
    if (p->score_kind != DASH_SCORE_REL && p->score_kind != DASH_SCORE_ABS) return DASH_ERR_INVALID_ARG;
    if (p->keep_first_n < 0 || p->keep_last_n < 0) return DASH_ERR_INVALID_ARG;
    if (p->rule == DASH_RULE_TOPK && p->k_keep < 0 && !(p->rho >= 0.0 && p->rho < 1.0))
        return DASH_ERR_INVALID_ARG;
    return DASH_OK;
}

struct Workspace {
    size_t o_off, partials_off, counts_off, decide_off, published_off, split_off, split_bytes, total;
};

Workspace carve(const dash_layer_params& p, int64_t n) {
    Workspace w;
    size_t off = 0;
    w.o_off = off;
    off = align_up(off + (size_t)n * p.n_q_heads * p.head_dim * elem_size(p.dtype), 256);
    w.partials_off = off;
    off = align_up(off + (size_t)n * norm_partials_per_row(p.d, p.dtype) * 2 * sizeof(float), 256);
    const size_t n_chunks = (size_t)(n + kChunkRows - 1) / kChunkRows;
    w.counts_off = off;
    off = align_up(off + n_chunks * sizeof(int32_t), 256);
    w.decide_off = off;
    off = align_up(off + decide_workspace_bytes() + n_chunks * sizeof(int32_t), 256);
    w.published_off = off;  // words of the fused score + decision + compaction kernel
    off = align_up(off + published_bytes((int)n), 256);
    w.split_off = off;
    w.split_bytes = wo_splitk_bytes(p, (int)n);  // split-K sums of the projection when few rows are active
    off += w.split_bytes;
    w.total = off;
    return w;
}

}  // namespace

extern "C" {

const char* dash_status_string(dash_status s) {
    switch (s) {
        case DASH_OK: return "ok";
        case DASH_ERR_INVALID_ARG: return "invalid argument";
        case DASH_ERR_UNSUPPORTED: return "unsupported shape or type";
        case DASH_ERR_WORKSPACE: return "workspace too small or misaligned";
        case DASH_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

const char* dash_version(void) { return "libdash 0.1 (gfx950)"; }

int64_t dash_keep_count(int64_t n, double rho, int32_t keep_first_n, int32_t keep_last_n,
                        int32_t paper_impl_rounding) {
    if (n < 0 || !(rho >= 0.0 && rho < 1.0) || keep_first_n < 0 || keep_last_n < 0) return -1;
    if (!paper_impl_rounding) {
        // Eq. 3 as n - ceil(rho n); a product within 1e-9 (relative) of a whole number counts as that number,
        // because the double of a decimal ratio (0.4, 0.667) sits a hair beside it
        double drop = rho * (double)n;
        const double whole = round(drop);
        if (fabs(drop - whole) <= 1e-9 * fmax(1.0, fabs(drop))) drop = whole;
        return n - (int64_t)ceil(drop);
    }
    const int64_t n_fix = (int64_t)keep_first_n + keep_last_n;
    if (n <= n_fix) return n;
    return n - llround(rho * (double)(n - n_fix));
}

int64_t dash_keep_count_quantile(int64_t n, double halt_frac) {
    if (n < 0 || !(halt_frac >= 0.0 && halt_frac <= 1.0)) return -1;
    return n - (int64_t)floor(halt_frac * (double)n);
}

double dash_block_cost(double n, double d, double m) {
    if (!(n >= 0.0) || !(d > 0.0) || !(m >= 0.0)) return -1.0;
    return 4.0 * n * d * d + 2.0 * n * n * d + 2.0 * n * d * m;
}

dash_status dash_schedule_lengths(int64_t n, int32_t L, const int32_t* shot_blocks, const double* shot_ratios,
                                  int32_t n_shots, int32_t keep_first_n, int32_t keep_last_n, int64_t* lengths) {
    if (n < 0 || L < 0 || n_shots < 0 || !lengths || keep_first_n < 0 || keep_last_n < 0) return DASH_ERR_INVALID_ARG;
    if (n_shots > 0 && (!shot_blocks || !shot_ratios)) return DASH_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_shots; ++i) {
        if (shot_blocks[i] < 0 || shot_blocks[i] >= L || (i > 0 && shot_blocks[i] <= shot_blocks[i - 1]))
            return DASH_ERR_INVALID_ARG;
        if (!(shot_ratios[i] >= 0.0 && shot_ratios[i] < 1.0)) return DASH_ERR_INVALID_ARG;
    }
    int64_t cur = n;
    int32_t next = 0;
    for (int32_t l = 0; l < L; ++l) {
        lengths[l] = cur;
        if (next < n_shots && shot_blocks[next] == l) {
            cur = dash_keep_count(cur, shot_ratios[next], keep_first_n, keep_last_n, 1);
            ++next;
        }
    }
    return DASH_OK;
}

double dash_schedule_cost(const int64_t* lengths, int32_t L, double d, double m) {
    if (!lengths || L < 0 || !(d > 0.0) || !(m >= 0.0)) return -1.0;
    double c = 0.0;
    for (int32_t l = 0; l < L; ++l) c += dash_block_cost((double)lengths[l], d, m);
    return c;
}

double dash_comparable_multi_shot_ratio(int64_t n, int32_t L, const int32_t* shot_blocks, int32_t n_shots,
                                        double target_cost, double d, double m, int32_t keep_first_n,
                                        int32_t keep_last_n, int32_t grid) {
    if (n < 0 || L <= 0 || L > 4096 || n_shots <= 0 || n_shots > L || !shot_blocks || grid <= 0) return -1.0;
    int64_t lengths[4096];
    double ratios[4096];
    // the cost falls (weakly) as the ratio grows: bisection for the smallest grid point within the budget
    auto cost = [&](int32_t i) {
        const double c = (double)i / (double)grid;
        for (int32_t s = 0; s < n_shots; ++s) ratios[s] = c;
        if (dash_schedule_lengths(n, L, shot_blocks, ratios, n_shots, keep_first_n, keep_last_n, lengths) != DASH_OK)
            return -1.0;
        return dash_schedule_cost(lengths, L, d, m);
    };
    int32_t lo = 0, hi = grid - 1;   // ratio 1 itself is not a valid compression ratio
    const double c_hi = cost(hi);
    if (c_hi < 0.0 || c_hi > target_cost) return -1.0;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (cost(mid) <= target_cost)
            hi = mid;
        else
            lo = mid + 1;
    }
    return (double)lo / (double)grid;
}

double dash_layer_flops(const dash_layer_params* p, int64_t n) {
    if (check_params(p) != DASH_OK || n < 0) return 0.0;
    const double nn = (double)n, Da = (double)p->n_q_heads * p->head_dim;
    const double pairs = p->causal ? nn * (nn + 1.0) / 2.0 : nn * nn;
    return 4.0 * p->head_dim * p->n_q_heads * pairs + 2.0 * nn * Da * (double)p->d;
}

int32_t dash_norm_partials_per_row(const dash_layer_params* p) {
    if (check_params(p) != DASH_OK) return 0;
    return norm_partials_per_row(p->d, p->dtype);
}

size_t dash_workspace_bytes(const dash_layer_params* p, int32_t n_capacity) {
    if (check_params(p) != DASH_OK || n_capacity < 0) return 0;
    return carve(*p, n_capacity).total;
}

dash_status dash_init(void) {
    dash_status st = init_flash_kernels();
    if (st != DASH_OK) return st;
    st = init_gemm_kernels();
    if (st != DASH_OK) return st;
    void* scratch = nullptr;
    return topk_static_scratch_ptr(&scratch);  // device address of the static TopK scratch on the current device
}

dash_profile* dash_profile_create(void) {
    dash_profile* pr = new (std::nothrow) dash_profile;
    if (!pr) return nullptr;
    pr->recorded = false;
    pr->merged = false;
    for (int i = 0; i <= DASH_N_STAGES; ++i) {
        if (hipEventCreate(&pr->ev[i]) != hipSuccess) {
            for (int k = 0; k < i; ++k) (void)hipEventDestroy(pr->ev[k]);
            delete pr;
            return nullptr;
        }
    }
    return pr;
}

void dash_profile_destroy(dash_profile* pr) {
    if (!pr) return;
    for (int i = 0; i <= DASH_N_STAGES; ++i) (void)hipEventDestroy(pr->ev[i]);
    delete pr;
}

dash_status dash_profile_read(dash_profile* pr, float* ms) {
    if (!pr || !ms || !pr->recorded) return DASH_ERR_INVALID_ARG;
    for (int i = 0; i < DASH_N_STAGES; ++i) {
        if (pr->merged && i == 2) {  // one launch for score, decision and compaction: reported as stage 3
            ms[2] = 0.f;
            DASH_HIP_CHECK(hipEventElapsedTime(&ms[3], pr->ev[2], pr->ev[4]));
            break;
        }
        DASH_HIP_CHECK(hipEventElapsedTime(&ms[i], pr->ev[i], pr->ev[i + 1]));
    }
    return DASH_OK;
}

dash_status dash_flash_fwd(const dash_layer_params* p, const void* q, const void* k, const void* v,
                           const int32_t* active_idx, int32_t n, void* o, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!q || !k || !v || !active_idx || !o) return DASH_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return DASH_ERR_INVALID_ARG;
    return launch_flash_fwd(*p, q, k, v, active_idx, n, o, nullptr, 0, (hipStream_t)hip_stream);
}

dash_status dash_wo_residual_rownorm(const dash_layer_params* p, const void* o, const void* w_o,
                                     const void* x, int32_t n, void* x_next, float* norm_partials,
                                     float* delta_dbg, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!o || !w_o || !x || !x_next || !norm_partials) return DASH_ERR_INVALID_ARG;
    if (!aligned16(o) || !aligned16(w_o) || !aligned16(x) || !aligned16(x_next) ||
        !aligned16(norm_partials) || !aligned16(delta_dbg) || !aligned16(workspace))
        return DASH_ERR_INVALID_ARG;
    // the scratch is optional here: without it the product is never split along K
    return launch_wo_residual_rownorm(*p, o, w_o, x, n, x_next, norm_partials, delta_dbg, workspace,
                                      workspace ? workspace_bytes : 0, (hipStream_t)hip_stream);
}

dash_status dash_score_decide(const dash_layer_params* p, const float* norm_partials, int32_t n,
                              float* scores, uint8_t* halt_mask, int32_t* chunk_keep_counts,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!norm_partials || !scores || !halt_mask || !chunk_keep_counts) return DASH_ERR_INVALID_ARG;
    if (!aligned16(norm_partials)) return DASH_ERR_INVALID_ARG;
    const size_t need = decide_workspace_bytes() + (size_t)((n + kChunkRows - 1) / kChunkRows) * 4;
    if (p->rule == DASH_RULE_TOPK && (!workspace || workspace_bytes < need || !aligned16(workspace)))
        return DASH_ERR_WORKSPACE;
    return launch_score_decide(*p, norm_partials, norm_partials_per_row(p->d, p->dtype), n, scores,
                               halt_mask, chunk_keep_counts, workspace, (hipStream_t)hip_stream);
}

dash_status dash_decide_topk(const dash_layer_params* p, const float* scores, int32_t n, int32_t keep_low,
                             uint8_t* halt_mask, int32_t* chunk_keep_counts, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!scores || !halt_mask || !chunk_keep_counts) return DASH_ERR_INVALID_ARG;
    if (p->k_keep < 0 && !(p->rho >= 0.0 && p->rho < 1.0)) return DASH_ERR_INVALID_ARG;
    const size_t need = decide_workspace_bytes() + (size_t)((n + kChunkRows - 1) / kChunkRows) * 4;
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return DASH_ERR_WORKSPACE;
    return launch_decide_topk(*p, scores, n, keep_low, halt_mask, chunk_keep_counts, workspace, true,
                              (hipStream_t)hip_stream);
}

dash_status dash_decide_topk_static(const dash_layer_params* p, const float* scores, int32_t n, int32_t keep_low,
                                    uint8_t* halt_mask, int32_t* chunk_keep_counts, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n > kStaticTopkMaxRows) return DASH_ERR_UNSUPPORTED;  // beyond what the static scratch holds
    if (n == 0) return DASH_OK;
    if (!scores || !halt_mask || !chunk_keep_counts) return DASH_ERR_INVALID_ARG;
    if (p->k_keep < 0 && !(p->rho >= 0.0 && p->rho < 1.0)) return DASH_ERR_INVALID_ARG;
    void* scratch = nullptr;
    st = topk_static_scratch_ptr(&scratch);
    if (st != DASH_OK) return st;
    // the kernels write the selection state and every tie count they later read, so nothing has to be cleared; this
    // entry point always takes the selection + flag kernels, which keep their state in the scratch
    return launch_decide_topk(*p, scores, n, keep_low, halt_mask, chunk_keep_counts, scratch, false,
                              (hipStream_t)hip_stream);
}

dash_status dash_score_diff_rows(const void* x_new, const void* x_old, int32_t n, int32_t d, int32_t dtype,
                                 int32_t score_kind, float* scores, void* hip_stream) {
    if (n < 0 || d <= 0 || (dtype != DASH_BF16 && dtype != DASH_F32)) return DASH_ERR_INVALID_ARG;
    if (score_kind != DASH_SCORE_REL && score_kind != DASH_SCORE_ABS) return DASH_ERR_INVALID_ARG;
    if (d % (dtype == DASH_BF16 ? 8 : 4) != 0) return DASH_ERR_UNSUPPORTED;
    if (n == 0) return DASH_OK;
    if (!x_new || !x_old || !scores || !aligned16(x_new) || !aligned16(x_old)) return DASH_ERR_INVALID_ARG;
    return launch_score_diff_rows(x_new, x_old, n, d, dtype, score_kind, scores, (hipStream_t)hip_stream);
}

dash_status dash_compact(const dash_layer_params* p, const uint8_t* halt_mask,
                         const int32_t* chunk_keep_counts, const int32_t* active_idx, const void* x_next,
                         int32_t n, void* x_compact, int32_t* new_active_idx, int32_t* n_active_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0 || !n_active_out) return DASH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n > 0) {
        if (!halt_mask || !active_idx || !x_next || !x_compact || !new_active_idx)
            return DASH_ERR_INVALID_ARG;
        if (!aligned16(x_next) || !aligned16(x_compact)) return DASH_ERR_INVALID_ARG;
        if (!chunk_keep_counts) {
            const size_t need = (size_t)((n + kChunkRows - 1) / kChunkRows) * 4;
            if (!workspace || workspace_bytes < need) return DASH_ERR_WORKSPACE;
            st = launch_chunk_counts(halt_mask, n, (int32_t*)workspace, s);
            if (st != DASH_OK) return st;
            chunk_keep_counts = (const int32_t*)workspace;
        }
    }
    return launch_compact(halt_mask, chunk_keep_counts, active_idx, x_next, n,
                          p->d * (int)elem_size(p->dtype), x_compact, new_active_idx, n_active_out, s);
}

dash_status dash_score_rows(const float* delta, const void* x, int32_t n, int32_t d, int32_t dtype,
                            int32_t score_kind, float* scores, void* hip_stream) {
    if (n < 0 || d <= 0 || d % 8 != 0) return DASH_ERR_INVALID_ARG;
    if (dtype != DASH_BF16 && dtype != DASH_F32) return DASH_ERR_INVALID_ARG;
    if (score_kind != DASH_SCORE_REL && score_kind != DASH_SCORE_ABS) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!delta || !scores || (score_kind == DASH_SCORE_REL && !x)) return DASH_ERR_INVALID_ARG;
    if (!aligned16(delta) || !aligned16(x)) return DASH_ERR_INVALID_ARG;
    return launch_score_rows(delta, x, n, d, dtype, score_kind, scores, (hipStream_t)hip_stream);
}

size_t dash_qkv_workspace_bytes(const dash_layer_params* p, int32_t n_capacity) {
    if (check_params(p) != DASH_OK || n_capacity < 0) return 0;
    return qkv_workspace_bytes(*p, n_capacity);
}

dash_status dash_rmsnorm_qkv(const dash_layer_params* p, const void* x, const void* w_q, const void* w_k,
                             const void* w_v, int32_t n, void* q, void* k, void* v, void* h_scratch,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (p->dtype != DASH_BF16) return DASH_ERR_UNSUPPORTED;
    if (p->d % 64 != 0) return DASH_ERR_UNSUPPORTED;  // K step of the projection GEMM
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!x || !w_q || !w_k || !w_v || !q || !k || !v || !h_scratch) return DASH_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_q) || !aligned16(w_k) || !aligned16(w_v) || !aligned16(q) ||
        !aligned16(k) || !aligned16(v) || !aligned16(h_scratch) || !aligned16(workspace))
        return DASH_ERR_INVALID_ARG;
    return launch_rmsnorm_qkv(*p, x, w_q, w_k, w_v, n, q, k, v, h_scratch, workspace,
                              workspace ? workspace_bytes : 0, (hipStream_t)hip_stream);
}

dash_status dash_rmsnorm_qkv_fused(const dash_layer_params* p, const void* x, const void* w_qkv, int32_t n, void* q,
                                   void* k, void* v, void* h_scratch, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (p->dtype != DASH_BF16) return DASH_ERR_UNSUPPORTED;
    if (p->d % 64 != 0) return DASH_ERR_UNSUPPORTED;  // K step of the projection GEMM
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!x || !w_qkv || !q || !k || !v || !h_scratch) return DASH_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_qkv) || !aligned16(q) || !aligned16(k) || !aligned16(v) ||
        !aligned16(h_scratch) || !aligned16(workspace))
        return DASH_ERR_INVALID_ARG;
    return launch_rmsnorm_qkv_fused(*p, x, w_qkv, n, q, k, v, h_scratch, workspace, workspace ? workspace_bytes : 0,
                                    (hipStream_t)hip_stream);
}

size_t dash_ffn_workspace_bytes(const dash_layer_params* p, int32_t n_capacity, int32_t m) {
    if (check_params(p) != DASH_OK || n_capacity < 0 || m <= 0) return 0;
    return ffn_workspace_bytes(*p, n_capacity, m);
}

dash_status dash_ffn_swiglu(const dash_layer_params* p, const void* x, const void* w_gate_up, const void* w_down,
                            int32_t n, int32_t m, void* x_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (p->dtype != DASH_BF16) return DASH_ERR_UNSUPPORTED;
    if (p->d % 64 != 0 || m <= 0 || m % 64 != 0) return DASH_ERR_UNSUPPORTED;  // K steps of the two GEMMs
    if (n < 0) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!x || !w_gate_up || !w_down || !x_out || !workspace) return DASH_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(w_gate_up) || !aligned16(w_down) || !aligned16(x_out) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return DASH_ERR_INVALID_ARG;
    if (workspace_bytes < ffn_workspace_bytes(*p, n, m)) return DASH_ERR_WORKSPACE;
    return launch_ffn_swiglu(*p, x, w_gate_up, w_down, n, m, x_out, workspace, (hipStream_t)hip_stream);
}

dash_status dash_scatter_rows(const void* rows, const int32_t* idx, const uint8_t* select, int32_t select_value,
                              int32_t n, int32_t d, int32_t dtype, int32_t N, void* full, void* hip_stream) {
    if (n < 0 || d <= 0 || N < 0 || (dtype != DASH_BF16 && dtype != DASH_F32)) return DASH_ERR_INVALID_ARG;
    if ((size_t)d * (dtype == DASH_BF16 ? 2 : 4) % 16 != 0) return DASH_ERR_UNSUPPORTED;
    if (n == 0) return DASH_OK;
    if (!rows || !idx || !full || !aligned16(rows) || !aligned16(full)) return DASH_ERR_INVALID_ARG;
    return launch_scatter_rows(rows, idx, select, select_value, n, d, dtype, N, full, (hipStream_t)hip_stream);
}

dash_status dash_rope_qk(const dash_layer_params* p, void* q, void* k, const int32_t* active_idx, int32_t n,
                         double theta_base, void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (p->dtype != DASH_BF16) return DASH_ERR_UNSUPPORTED;
    if (n < 0 || !(theta_base > 1.0)) return DASH_ERR_INVALID_ARG;
    if (n == 0) return DASH_OK;
    if (!q || !k || !active_idx || !aligned16(q) || !aligned16(k)) return DASH_ERR_INVALID_ARG;
    return launch_rope_qk(*p, q, k, active_idx, n, theta_base, (hipStream_t)hip_stream);
}

double dash_mfma_probe_flops(int32_t iters, int32_t workgroups) {
    if (iters <= 0 || workgroups <= 0) return 0.0;
    return 524288.0 * (double)iters * 8.0 * (double)workgroups;  // per iteration and wave, 8 waves per workgroup
}

dash_status dash_mfma_probe(int32_t shape, int32_t normal_data, int32_t iters, int32_t workgroups, float* sink,
                            void* hip_stream) {
    if ((shape != 0 && shape != 1) || iters <= 0 || workgroups <= 0 || workgroups > 65536 || !sink)
        return DASH_ERR_INVALID_ARG;
    return launch_mfma_probe(shape == 0, normal_data != 0, iters, workgroups, sink, (hipStream_t)hip_stream);
}

dash_status dash_validate_active_idx(const int32_t* active_idx, int32_t n, int32_t N, int32_t* violations,
                                     void* hip_stream) {
    if (n < 0 || !violations || (n > 0 && !active_idx)) return DASH_ERR_INVALID_ARG;
    return launch_validate_idx(active_idx, n, N, violations, (hipStream_t)hip_stream);
}

dash_status dash_attn_layer(const dash_layer_params* p, const void* x, const void* q, const void* k,
                            const void* v, const void* w_o, const int32_t* active_idx, int32_t n,
                            void* x_next, float* scores, uint8_t* halt_mask, void* x_compact,
                            int32_t* new_active_idx, int32_t* n_active_out, float* delta_dbg,
                            void* workspace, size_t workspace_bytes, dash_profile* profile,
                            void* hip_stream) {
    dash_status st = check_params(p);
    if (st != DASH_OK) return st;
    if (n < 0 || !n_active_out) return DASH_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n == 0)
        return launch_compact(nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, n_active_out, s);
    if (!x || !q || !k || !v || !w_o || !active_idx || !x_next || !scores || !halt_mask || !x_compact ||
        !new_active_idx)
        return DASH_ERR_INVALID_ARG;
    const void* ptrs[] = {x, q, k, v, w_o, x_next, x_compact, delta_dbg};
    for (const void* ptr : ptrs)
        if (!aligned16(ptr)) return DASH_ERR_INVALID_ARG;
    const Workspace w = carve(*p, n);
    if (!workspace || workspace_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return DASH_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    void* o = ws + w.o_off;
    float* partials = reinterpret_cast<float*>(ws + w.partials_off);
    int32_t* counts = reinterpret_cast<int32_t*>(ws + w.counts_off);
    void* decide_ws = ws + w.decide_off;

    // NONE / THRESHOLD: scores, decision and compaction run as one launch whose workgroups hand each other the
    // chunks' kept masks through words that have to start cleared: the attention kernel clears them on its way
    const bool one_launch = p->rule != DASH_RULE_TOPK;
    uint32_t* published = reinterpret_cast<uint32_t*>(ws + w.published_off);
    const int n_clear = one_launch ? (int)(published_bytes(n) / sizeof(uint32_t)) : 0;
    if (profile) DASH_HIP_CHECK(hipEventRecord(profile->ev[0], s));
    st = launch_flash_fwd(*p, q, k, v, active_idx, n, o, published, n_clear, s);
    if (st != DASH_OK) return st;
    if (profile) DASH_HIP_CHECK(hipEventRecord(profile->ev[1], s));
    st = launch_wo_residual_rownorm(*p, o, w_o, x, n, x_next, partials, delta_dbg, ws + w.split_off, w.split_bytes, s);
    if (st != DASH_OK) return st;
    if (profile) DASH_HIP_CHECK(hipEventRecord(profile->ev[2], s));
    if (one_launch) {
        st = launch_score_decide_compact(*p, partials, norm_partials_per_row(p->d, p->dtype), n, scores, halt_mask,
                                         published, active_idx, x_next, p->d * (int)elem_size(p->dtype), x_compact,
                                         new_active_idx, n_active_out, s);
    } else {
        st = launch_score_decide(*p, partials, norm_partials_per_row(p->d, p->dtype), n, scores, halt_mask,
                                 counts, decide_ws, s);
        if (st != DASH_OK) return st;
        if (profile) DASH_HIP_CHECK(hipEventRecord(profile->ev[3], s));
        st = launch_compact(halt_mask, counts, active_idx, x_next, n, p->d * (int)elem_size(p->dtype), x_compact,
                            new_active_idx, n_active_out, s);
    }
    if (st != DASH_OK) return st;
    if (profile) {
        DASH_HIP_CHECK(hipEventRecord(profile->ev[4], s));
        profile->recorded = true;
        profile->merged = one_launch;
    }
    return DASH_OK;
}

}  // extern "C"
