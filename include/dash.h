/*
 * libdash: the hot path of DASH (Delta Attention Selective Halting) for one GPU (gfx950).
 *
 * One prefill self-attention layer executed over only the still-active tokens
 * (Sec. 3.4: every block runs on the compacted active sequence), followed by the
 * per-token delta-attention score (Eq. 2), the halting decision (Eq. 3) and the
 * stream compaction that hands the next layer a shorter sequence (Alg. 1 step 4).
 *
 * Conventions for every entry point
 *   - Plain C ABI. Pointers marked "device" are GPU global memory owned by the
 *     caller; "host" pointers are ordinary host memory. The compute entry points
 *     allocate nothing: every buffer, the workspaces included, is the caller's.
 *     What the library does keep: (i) per process, the number of compute units of the
 *     device and the one-time launch attributes of its kernels, set by dash_init() or
 *     by the first call that needs them (call dash_init() before capturing calls in
 *     a HIP graph); (ii) dash_profile objects, the only thing it allocates (host
 *     memory and HIP events, created and destroyed by the caller through
 *     dash_profile_create / dash_profile_destroy). Results never depend on either.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); calls return after enqueue and never synchronise.
 *   - Every device pointer must be 16-byte aligned. Matrices are row-major and
 *     dense (no padding between rows).
 *   - Errors are reported as a dash_status; argument errors are found on the host
 *     before anything is launched, HIP launch errors map to DASH_ERR_HIP.
 *   - Largest sizes. Row counts are int32 and addresses are formed in 64 bits; two kernels
 *     add 32-bit byte offsets to a 64-bit base, which bounds what they accept (larger
 *     arguments return DASH_ERR_UNSUPPORTED, nothing is launched): attention with bf16
 *     storage needs n * Hkv * dh * 2 < 2^31 bytes of K (2 097 151 rows at Hkv * dh = 512,
 *     1 048 575 at 1024); the bf16 products need 256 * K * 2 < 2^32 and 64 * N * 2 + 512 <
 *     2^32 for a [M,K] x [K,N] product (any M). dash_decide_topk_static has its own row limit.
 *   - dtype selects the storage type of x, q, k, v, w_o, O, x_next, x_compact:
 *     DASH_BF16 (MFMA kernels, fp32 accumulation and fp32 softmax) or DASH_F32
 *     (plain fp32 kernels). Scores and norm partials are always fp32.
 */
#ifndef DASH_H
#define DASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DASH_OK = 0,
    DASH_ERR_INVALID_ARG = -1,
    DASH_ERR_UNSUPPORTED = -2,
    DASH_ERR_WORKSPACE = -3,
    DASH_ERR_HIP = -4
} dash_status;

typedef enum { DASH_BF16 = 0, DASH_F32 = 1 } dash_dtype;

/* NONE: no token halts (layers before the start layer l_s of the single-shot
 * schedule, Sec. 3.2); scores are still produced. THRESHOLD: the cut drawn as a
 * threshold line in Fig. 8. TOPK: Eq. 3. */
typedef enum { DASH_RULE_NONE = 0, DASH_RULE_THRESHOLD = 1, DASH_RULE_TOPK = 2 } dash_rule;

/* REL: ||U_t||_2 / max(||H_t||_2, 1e-30), H_t the row entering the block (the
 * "relative" delta-attention of Fig. 1). ABS: ||U_t||_2 (Eq. 2). */
typedef enum { DASH_SCORE_REL = 0, DASH_SCORE_ABS = 1 } dash_score_kind;

typedef struct {
    int32_t d;            /* hidden size (columns of x and of w_o) */
    int32_t n_q_heads;    /* query heads; n_q_heads * head_dim = rows of w_o */
    int32_t n_kv_heads;   /* key/value heads; must divide n_q_heads */
    int32_t head_dim;     /* 64 or 128 */
    int32_t dtype;        /* dash_dtype */
    int32_t causal;       /* non-zero: key j visible to query i iff its original position
                             active_idx[j] <= active_idx[i] */
    float softmax_scale;  /* <= 0 selects 1/sqrt(head_dim) */
    int32_t rule;         /* dash_rule */
    int32_t score_kind;   /* dash_score_kind */
    float tau;            /* THRESHOLD: a row halts iff score < tau (equal or NaN is kept) */
    int32_t k_keep;       /* TOPK: rows kept in total, protected rows included;
                             < 0 selects floor((1 - rho) * n_active)  (Eq. 3) */
    double rho;           /* pruning ratio in [0,1), used only when k_keep < 0; a double, so that the rows kept
                             are exactly dash_keep_count(n_active, rho, 0, 0, 0) for the caller's rho */
    int32_t keep_first_n; /* protected ranks at the head of the current active order (App. A) */
    int32_t keep_last_n;  /* protected ranks at its tail; protected rows never halt */
} dash_layer_params;

/* Optional per-stage timing. When a dash_profile is passed to dash_attn_layer it
 * records HIP events on the launch stream around the four stages; read them back
 * with dash_profile_read after the stream has been synchronised by the caller. */
typedef struct dash_profile dash_profile;
#define DASH_N_STAGES 4 /* 0 flash attention, 1 W_o+residual+norms, 2 score+decision, 3 compaction. Under the rules
                           NONE and THRESHOLD stages 2 and 3 are one launch: its time is reported as stage 3, stage 2 as 0 */

/* One-time set-up on the current device: reads the device's compute-unit count and sets the launch attributes of
 * the kernels (their LDS sizes) and looks up the device address of the static scratch of dash_decide_topk_static.
 * Optional: the first compute call that needs one of these does the same. Synchronous, host; launches
 * nothing. Returns DASH_ERR_HIP when there is no usable device. */
dash_status dash_init(void);

dash_profile *dash_profile_create(void);            /* host; NULL on failure */
void dash_profile_destroy(dash_profile *);          /* host */
/* host; ms[DASH_N_STAGES] receives the stage durations of the LAST profiled call.
 * The stream must be idle (caller synchronised). */
dash_status dash_profile_read(dash_profile *, float *ms);

/* Bytes of device workspace dash_attn_layer needs for up to n_capacity active rows
 * (0 on invalid params). Host. */
size_t dash_workspace_bytes(const dash_layer_params *params, int32_t n_capacity);

/* Number of fp32 (sum delta^2, sum x^2) pairs per row that the projection stage
 * writes and the score stage reads; depends only on params->d and dtype. Host. */
int32_t dash_norm_partials_per_row(const dash_layer_params *params);

/*
 * The whole layer step on the active rows (Eq. 1-3, Alg. 1 steps 4-6 and 9-13):
 *   O      = Attn(q, k, v)                    causal GQA softmax attention
 *   delta  = O * w_o                          U of Eq. 1 (before the residual add)
 *   x_next = x + delta                        for ALL n_active rows, halted-now rows included
 *   scores = ||delta_t|| [/ ||x_t||]          Eq. 2 from the fp32 accumulators
 *   halt   = decision(scores)                 params->rule
 *   new_active_idx, x_compact, n_active_out = stable compaction of the kept rows
 *
 * device inputs : x [n,d], q [n,Hq,dh], k,v [n,Hkv,dh], w_o [Hq*dh, d] (delta = O @ w_o),
 *                 active_idx [n] int32, strictly increasing original positions
 * host input    : n_active (rows), >= 0; 0 is a valid no-op that writes n_active_out = 0
 * device outputs: x_next [n,d]; scores [n] fp32; halt_mask [n] uint8 (1 = halted);
 *                 x_compact [n,d] (first n_active_out rows valid, bitwise copies of kept
 *                 x_next rows); new_active_idx [n] (first n_active_out valid);
 *                 n_active_out: ONE device int32
 *                 delta_dbg: NULL, or fp32 [n,d] that receives delta
 * workspace     : device, >= dash_workspace_bytes(params, n_active), 256-byte aligned
 * profile       : NULL or a dash_profile
 *
 * active_idx is trusted, not checked: a check would put a pass over n values and a read-back on the path of
 * every layer. Its values are only compared with each other (the causal mask of tiles on the diagonal), turned
 * into rotation angles (dash_rope_qk) and copied to new_active_idx, never used as addresses, so a list that is
 * not strictly increasing gives a mask that means nothing but no access out of bounds.
 * dash_validate_active_idx is the check, for callers that build the list themselves.
 * The call records kernels only (no memset, no copy, no allocation), so it can be captured in a HIP graph once
 * dash_init() has run on the device.
 */
dash_status dash_attn_layer(const dash_layer_params *params, const void *x, const void *q, const void *k,
                            const void *v, const void *w_o, const int32_t *active_idx, int32_t n_active,
                            void *x_next, float *scores, uint8_t *halt_mask, void *x_compact,
                            int32_t *new_active_idx, int32_t *n_active_out, float *delta_dbg,
                            void *workspace, size_t workspace_bytes, dash_profile *profile,
                            void *hip_stream);

/* ---- stage-level entry points (same conventions), so each kernel can be tested and timed alone ---- */

/* Stage 0. Attention of Eq. 1 without the output projection: o [n, Hq*dh] in params->dtype.
 * Tiled online-softmax forward; the probability matrix never reaches HBM. */
dash_status dash_flash_fwd(const dash_layer_params *params, const void *q, const void *k, const void *v,
                           const int32_t *active_idx, int32_t n_active, void *o, void *hip_stream);

/* Stage 1. delta = o @ w_o; x_next = x + delta (Sec. 3.1, Alg. 1 step 6); per-row partial sums of
 * delta^2 and x^2 taken from the fp32 accumulators: norm_partials [P, n, 2] fp32 (P-major) with
 * P = dash_norm_partials_per_row(params). delta_dbg NULL or fp32 [n,d].
 * workspace: optional device scratch (NULL or 16-byte aligned). With few active rows the product has few
 * output tiles; given scratch it is then cut along the contraction into parts that run side by side and
 * are summed in a fixed order (as many parts as the scratch holds fp32 [n,d] sums; dash_workspace_bytes
 * reserves enough for dash_attn_layer). Results do not depend on other calls, only on n and the scratch size. */
dash_status dash_wo_residual_rownorm(const dash_layer_params *params, const void *o, const void *w_o,
                                     const void *x, int32_t n, void *x_next, float *norm_partials,
                                     float *delta_dbg, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/* Stage 2. scores (Eq. 2) from the partials, then the decision (Eq. 3 / threshold).
 * chunk_keep_counts: device int32 [ceil(n/64)], kept rows per 64-row chunk, consumed by dash_compact.
 * workspace: device scratch, needed for TOPK only: >= 256 + 4*ceil(n/64) bytes, 16-byte aligned
 * (selection state and tie counts). */
dash_status dash_score_decide(const dash_layer_params *params, const float *norm_partials, int32_t n,
                              float *scores, uint8_t *halt_mask, int32_t *chunk_keep_counts,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Stage 3. Stable stream compaction by halt_mask (Alg. 1 step 4): prefix sum of kept flags, gather of
 * hidden rows and original positions. chunk_keep_counts as written by dash_score_decide, or NULL to
 * have them recomputed from halt_mask into workspace (>= 4*ceil(n/64) bytes). */
dash_status dash_compact(const dash_layer_params *params, const uint8_t *halt_mask,
                         const int32_t *chunk_keep_counts, const int32_t *active_idx, const void *x_next,
                         int32_t n, void *x_compact, int32_t *new_active_idx, int32_t *n_active_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Standalone score of Eq. 2 from a stored fp32 delta [n,d] and x [n,d] (dtype): one pass over HBM. */
dash_status dash_score_rows(const float *delta, const void *x, int32_t n, int32_t d, int32_t dtype,
                            int32_t score_kind, float *scores, void *hip_stream);

/* Variants of the ablation (Sec. 5.4), built from the same decision and compaction kernels:
 *  - dash_score_diff_rows: the block-level signal, Eq. 2 applied to the change of a row across a whole block,
 *    ||x_new_t - x_old_t||_2 [/ ||x_old_t||_2] (x_new, x_old: device [n,d] in dtype; one pass over HBM).
 *  - dash_decide_topk: the TopK decision of Eq. 3 on scores the caller provides (device fp32 [n]): any signal,
 *    or random numbers for the random-halting control. keep_low != 0 keeps the K LOWEST scores instead (the
 *    high-Delta tokens halt: the direction control). K, rho and the protected ranges come from params as for
 *    DASH_RULE_TOPK; ties keep the earlier row. Outputs and workspace as in dash_score_decide. */
dash_status dash_score_diff_rows(const void *x_new, const void *x_old, int32_t n, int32_t d, int32_t dtype,
                                 int32_t score_kind, float *scores, void *hip_stream);
dash_status dash_decide_topk(const dash_layer_params *params, const float *scores, int32_t n, int32_t keep_low,
                             uint8_t *halt_mask, int32_t *chunk_keep_counts, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* dash_decide_topk for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. Same decision, same outputs (bit for bit), no workspace argument:
 * the selection state and tie counts live in a device array that is part of the library image
 * (256 + 4 * DASH_TOPK_STATIC_MAX_ROWS / 64 bytes = 65 792 bytes on every GPU the library runs on, held until the
 * process ends). Allocates nothing and frees nothing. n > DASH_TOPK_STATIC_MAX_ROWS returns DASH_ERR_UNSUPPORTED.
 * It runs the selection and flag kernels at every size (dash_decide_topk takes a one-launch kernel that needs no
 * scratch up to 16384 rows, 1-2 us faster there).
 * The first call on a device (or dash_init() with that device current) looks up the array's device address; do
 * that outside a graph capture. All calls on one GPU share that GPU's array, which keeps the last call's contents
 * (the kernels overwrite what they read, nothing needs clearing): calls that overlap on one GPU (different
 * streams, or threads) race; calls on one stream are ordered and safe. */
#define DASH_TOPK_STATIC_MAX_ROWS (1 << 20)
dash_status dash_decide_topk_static(const dash_layer_params *params, const float *scores, int32_t n,
                                    int32_t keep_low, uint8_t *halt_mask, int32_t *chunk_keep_counts,
                                    void *hip_stream);

/* Front end of a layer in a chain (Eq. 1's LN and the q/k/v projections, which sit before the path):
 * h = x / sqrt(mean(x^2) + 1e-6) (unit gain); q = h @ w_q [d, Hq*dh]; k = h @ w_k; v = h @ w_v
 * [d, Hkv*dh]. bf16 only. h_scratch: device [n,d] bf16.
 * workspace: optional device scratch (NULL or 16-byte aligned) of dash_qkv_workspace_bytes(params, n_capacity)
 * bytes, which lets the projections of a short active sequence split along the contraction (see
 * dash_wo_residual_rownorm). */
size_t dash_qkv_workspace_bytes(const dash_layer_params *params, int32_t n_capacity);
dash_status dash_rmsnorm_qkv(const dash_layer_params *params, const void *x, const void *w_q,
                             const void *w_k, const void *w_v, int32_t n, void *q, void *k, void *v,
                             void *h_scratch, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same front end as ONE product over the concatenated weight w_qkv = [w_q | w_k | w_v], device
 * [d, (Hq + 2 Hkv) * dh] row-major: the normalised rows are read once instead of three times and the narrow k and
 * v projections no longer run as launches of their own. Outputs, scratch and workspace as in dash_rmsnorm_qkv. */
dash_status dash_rmsnorm_qkv_fused(const dash_layer_params *params, const void *x, const void *w_qkv, int32_t n,
                                   void *q, void *k, void *v, void *h_scratch, void *workspace,
                                   size_t workspace_bytes, void *hip_stream);

/* Rotary position embedding of the backbone (Qwen2.5 / Llama-3, Sec. 4.1) applied in place to q [n,Hq,dh] and
 * k [n,Hkv,dh] (bf16, device), with each row's ORIGINAL position active_idx[t]: the compacted active sequence
 * of Sec. 3.4 keeps the position ids, so this is where active_idx matters numerically. "Rotate-half" pairing:
 * for i < dh/2 and a = active_idx[t] * theta_base^(-2i/dh):
 *   u[i], u[i+dh/2] <- u[i] cos a - u[i+dh/2] sin a, u[i] sin a + u[i+dh/2] cos a.
 * theta_base > 1 (1e6 for Qwen2.5, 5e5 for Llama-3). Part of the front end, like dash_rmsnorm_qkv. */
dash_status dash_rope_qk(const dash_layer_params *params, void *q, void *k, const int32_t *active_idx, int32_t n,
                         double theta_base, void *hip_stream);

/* Second half of a block (Alg. 1 step 7): x_out = x + FFN(LN(x)) on n rows, LN = RMS normalisation (unit gain,
 * eps 1e-6), FFN the gated feed-forward of the Qwen2.5 / Llama-3 backbones (Sec. 4.1):
 *   h = LN(x); a = silu(h W_gate) * (h W_up); x_out = x + a W_down.
 * bf16 only; d % 64 == 0, m % 64 == 0. device: x, x_out [n,d] (x_out may be x); w_down [m,d];
 * w_gate_up [d, 2m]: W_gate and W_up interleaved in blocks of 32 columns - columns 64c..64c+31 are columns
 * 32c..32c+31 of W_gate, columns 64c+32..64c+63 the same columns of W_up (so that one GEMM tile holds gate and
 * up of the same features and the gating happens in its epilogue).
 * workspace: device, 256-byte aligned, >= dash_ffn_workspace_bytes(params, n, m) (the normalised rows, the
 * gated activations [n,m], row-norm partials, split sums of the two products when n is small). */
size_t dash_ffn_workspace_bytes(const dash_layer_params *params, int32_t n_capacity, int32_t m);
dash_status dash_ffn_swiglu(const dash_layer_params *params, const void *x, const void *w_gate_up,
                            const void *w_down, int32_t n, int32_t m, void *x_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* Halted tokens keep the state they had when they halted (Sec. 3.4): full[idx[t], :] = rows[t, :] for every t with
 * select == NULL or select[t] == select_value (e.g. select = halt_mask, select_value = 1: the rows that halt now).
 * device: rows [n,d], idx [n] original positions, select [n] uint8 or NULL, full [N,d]; dtype as dash_dtype; row
 * bytes must be a multiple of 16. Rows whose position lies outside [0, N) are skipped. */
dash_status dash_scatter_rows(const void *rows, const int32_t *idx, const uint8_t *select, int32_t select_value,
                              int32_t n, int32_t d, int32_t dtype, int32_t N, void *full, void *hip_stream);

/* Debug aid: counts rows where active_idx is not strictly increasing or lies outside [0, N)
 * (N < 0: no upper bound) into ONE device int32 *violations. */
dash_status dash_validate_active_idx(const int32_t *active_idx, int32_t n, int32_t N, int32_t *violations,
                                     void *hip_stream);

/* Measurement aid (no step of the method): a register-only loop of independent bf16 MFMAs, 8 waves per workgroup,
 * no memory or LDS traffic, to read what the matrix pipe sustains on this part beside the published peak.
 * shape 0: v_mfma_f32_32x32x16_bf16 (the attention kernel's), 1: v_mfma_f32_16x16x32_bf16 (the GEMMs');
 * normal_data 0: all operands zero, else N(0,1) values as in the workloads (the part lowers its clock under the
 * power the operand bits draw). Runs `iters` iterations in each of `workgroups` workgroups (use the number of
 * compute units); sink: device fp32 [workgroups * 512], written once at the end. The caller times the launch;
 * dash_mfma_probe_flops(iters, workgroups) is the flop count of one launch. */
dash_status dash_mfma_probe(int32_t shape, int32_t normal_data, int32_t iters, int32_t workgroups, float *sink,
                            void *hip_stream);
double dash_mfma_probe_flops(int32_t iters, int32_t workgroups);

/* Host arithmetic: tokens kept out of n.
 * paper_impl_rounding == 0: floor((1 - rho) n) (Eq. 3), evaluated as n - ceil(rho n) with a product that lies
 * within 1e-9 (relative) of a whole number taken as that number, so that decimal ratios give what exact
 * arithmetic on the decimal gives (rho = 0.667, n = 1000 keeps 333);
 * otherwise n - round(rho * (n - keep_first_n - keep_last_n)) (App. A, caption of Table 5).
 * Returns -1 on invalid arguments. */
int64_t dash_keep_count(int64_t n, double rho, int32_t keep_first_n, int32_t keep_last_n,
                        int32_t paper_impl_rounding);

/* Host arithmetic: rows kept when the h = floor(halt_frac * n) lowest-scoring rows halt (a cut at the halt_frac
 * quantile of the scores, the TopK equivalent of a threshold drawn at that quantile as in Fig. 8): n - h.
 * halt_frac in [0,1]; returns -1 on invalid arguments. */
int64_t dash_keep_count_quantile(int64_t n, double halt_frac);

/* Host arithmetic of the prefill cost model (App. A).
 *  - dash_block_cost: the per-block proxy A(n) = 4 n d^2 + 2 n^2 d + 2 n d m (Eq. 4), d hidden size, m FFN width.
 *  - dash_schedule_lengths: lengths[l] = rows block l runs on, l = 0..L-1, for a prompt of n tokens when halting
 *    decisions are taken after the blocks shot_blocks[0..n_shots) (strictly increasing, each in [0, L)) with
 *    compression ratios shot_ratios[i]: the deciding block still runs on all rows that enter it (Alg. 1 takes the
 *    decision after the block's FFN), the blocks after it on dash_keep_count(rows, ratio, keep_first_n,
 *    keep_last_n, 1) rows (App. A's rule on the current length). One shot at l_s is the single-shot schedule.
 *  - dash_schedule_cost: sum over the blocks of A(lengths[l]); for one shot this is l_s A(n) + (L - l_s) A(n^)
 *    (Eq. 6-7 with C_full = dash_schedule_cost of the schedule without shots).
 *  - dash_comparable_multi_shot_ratio: the smallest ratio c = i / grid (i = 0..grid) such that the schedule
 *    that applies c at every block of shot_blocks costs no more than target_cost (App. D compares single- and
 *    multi-shot selection "under comparable budgets" without giving the split; this is the reading taken).
 *    Returns -1 when no ratio on the grid meets the budget or on invalid arguments.
 * dash_schedule_lengths returns DASH_ERR_INVALID_ARG for bad arguments; the cost functions return -1. */
double dash_block_cost(double n, double d, double m);
dash_status dash_schedule_lengths(int64_t n, int32_t L, const int32_t *shot_blocks, const double *shot_ratios,
                                  int32_t n_shots, int32_t keep_first_n, int32_t keep_last_n, int64_t *lengths);
double dash_schedule_cost(const int64_t *lengths, int32_t L, double d, double m);
double dash_comparable_multi_shot_ratio(int64_t n, int32_t L, const int32_t *shot_blocks, int32_t n_shots,
                                        double target_cost, double d, double m, int32_t keep_first_n,
                                        int32_t keep_last_n, int32_t grid);

/* Algorithmic floating-point operations of stages 0+1 for n active rows: causal triangle
 * 4*dh*Hq*n(n+1)/2 (or the full square when not causal) plus 2*n*(Hq*dh)*d. Host. */
double dash_layer_flops(const dash_layer_params *params, int64_t n);

const char *dash_status_string(dash_status);
const char *dash_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DASH_H */
