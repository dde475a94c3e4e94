/*
 * DASH reference oracle: a slow, plain fp64 CPU implementation of one prefill
 * self-attention layer run over the still-active tokens, the per-token
 * delta-attention score, the halting decision and the stream compaction.
 *
 * THIS IS TEST INFRASTRUCTURE. It exists so that the GPU library can be checked
 * against something written straight from the paper. Only the test-suite, the
 * smoke check and the CPU-baseline leg of the benchmark may call it; the product
 * path never does. It shares no code with the GPU library.
 *
 * Every function walks the definition in the order the paper gives it, with no
 * blocking, fusion or reordering, so it can be compared with the paper by eye:
 *
 *   - attention_rows     : U = Attn(.) of Eq. 1 before the output projection;
 *                          textbook causal softmax attention with grouped KV
 *                          heads, causality decided on ORIGINAL token positions
 *                          (Sec. 3.4: blocks run on the compacted active sequence)
 *   - rmsnorm            : the LN of Eq. 1 as unit-gain RMS normalisation (front end
 *                          of a layer chain; sits before the path proper)
 *   - rope               : rotary position embedding of the backbone applied to q and k
 *                          with each token's ORIGINAL position (Sec. 3.4: the compacted
 *                          sequence keeps the position ids); front end, before the path
 *   - ffn_swiglu         : H^(l+1) = H~ + FFN(LN(H~)) (Alg. 1 step 7) with the gated FFN of the
 *                          Qwen2.5 / Llama-3 backbones: (silu(h W_gate) * (h W_up)) W_down
 *   - scatter_rows       : halted tokens keep their last updated state (Sec. 3.4): rows written
 *                          back to a full-length buffer at their original positions
 *   - project            : the output projection that completes U (Sec. 3.1:
 *                          U is the attention output before the residual add)
 *   - residual           : H~ = H + U                  (Sec. 3.1, Alg. 1 step 6)
 *   - scores             : Delta_t = ||U_t||_2         (Eq. 2), optionally
 *                          divided by ||H_t||_2 (the "relative" form of Fig. 1)
 *   - decide_topk        : S* = TopK(S, K, Delta)      (Eq. 3): keep high, halt low
 *   - decide_threshold   : the threshold-line form of the same cut (Fig. 8)
 *   - decide_topk_keep_low : the direction control of Sec. 5.4 (high-Delta tokens halt)
 *   - compact            : gather rows by the surviving index set
 *                          (Alg. 1 step 4, Sec. 3.4)
 *   - keep_count         : K = floor((1-rho) T) (Eq. 3) and the kept length
 *                          n^ of App. A (Eq. 5 with the rounding of Table 5)
 *   - flops_A / flops_*  : App. A, Eq. 4-9
 *
 * Pins (see the CPU tests): brute-force attention on tiny inputs, closed forms
 * (equal keys -> running mean of V; n = 1), exact identities (x_next - x = U,
 * W_o = 0 -> score 0, W_o = I), row-scaling covariance of the relative score,
 * hand-made decision vectors, the kept lengths and FLOPs ratios of Table 5.
 * Task-level accuracy of the paper pins nothing here: parity unpinned at task
 * level (needs the paper's weights and datasets).
 *
 * All arrays are row-major fp64 unless stated; sizes are element counts.
 * Return value: 0 on success, negative on invalid arguments.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_SCORE_REL 0
#define ORACLE_SCORE_ABS 1
/* Floor on the denominator of the relative score: a zero input row with a
 * non-zero update gets a huge score (kept); 0/eps = 0. */
#define ORACLE_NORM_EPS 1e-30

int dash_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention for a list of query rows against ALL keys/values (Eq. 1, Attn).
 *   q   [n, Hq, dh]    k, v [n, Hkv, dh]    pos [n] original positions
 *   rows[n_rows]       indices into 0..n-1 of the query rows wanted
 *   out [n_rows, Hq*dh]
 * Query head h reads KV head h / (Hq/Hkv). Key j is visible to query i when
 * pos[j] <= pos[i] (causal) or always (non-causal).
 * softmax_j(l_j) = exp(l_j - max) / sum exp(l_j - max), l_j = scale * <q_i, k_j>.
 */
int dash_oracle_attention_rows(const double *q, const double *k, const double *v,
                               const int32_t *pos, int64_t n, int32_t Hq, int32_t Hkv,
                               int32_t dh, int32_t causal, double scale,
                               const int64_t *rows, int64_t n_rows, double *out) {
    if (!q || !k || !v || !pos || !rows || !out) return -1;
    if (n <= 0 || Hq <= 0 || Hkv <= 0 || dh <= 0 || Hq % Hkv != 0 || n_rows < 0) return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= n) return -1;
    const int32_t group = Hq / Hkv;
    const int64_t tasks = n_rows * (int64_t)Hq;
    int failed = 0;
#pragma omp parallel
    {
        double *logit = (double *)malloc((size_t)n * sizeof(double));
        if (!logit) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t t = 0; t < tasks; ++t) {
                const int64_t r = t / Hq;
                const int32_t h = (int32_t)(t % Hq);
                const int64_t i = rows[r];
                const int32_t g = h / group;
                const double *qi = q + ((size_t)i * Hq + h) * dh;
                double *o = out + ((size_t)r * Hq + h) * dh;
                double mx = -INFINITY;
                for (int64_t j = 0; j < n; ++j) {
                    if (causal && pos[j] > pos[i]) continue;
                    const double *kj = k + ((size_t)j * Hkv + g) * dh;
                    double dot = 0.0;
                    for (int32_t c = 0; c < dh; ++c) dot += qi[c] * kj[c];
                    logit[j] = dot * scale;
                    if (logit[j] > mx) mx = logit[j];
                }
                double denom = 0.0;
                for (int64_t j = 0; j < n; ++j) {
                    if (causal && pos[j] > pos[i]) continue;
                    denom += exp(logit[j] - mx);
                }
                for (int32_t c = 0; c < dh; ++c) o[c] = 0.0;
                for (int64_t j = 0; j < n; ++j) {
                    if (causal && pos[j] > pos[i]) continue;
                    const double p = exp(logit[j] - mx) / denom;
                    const double *vj = v + ((size_t)j * Hkv + g) * dh;
                    for (int32_t c = 0; c < dh; ++c) o[c] += p * vj[c];
                }
            }
        }
        free(logit);
    }
    return failed ? -2 : 0;
}

/* U = O * W_o.   O [m, Da], w_o [Da, d] row-major, delta [m, d]. */
int dash_oracle_project(const double *O, const double *w_o, int64_t m, int32_t Da, int32_t d,
                        double *delta) {
    if (!O || !w_o || !delta || m < 0 || Da <= 0 || d <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double *di = delta + (size_t)i * d;
        for (int32_t c = 0; c < d; ++c) di[c] = 0.0;
        for (int32_t a = 0; a < Da; ++a) {
            const double oa = O[(size_t)i * Da + a];
            const double *wr = w_o + (size_t)a * d;
            for (int32_t c = 0; c < d; ++c) di[c] += oa * wr[c];
        }
    }
    return 0;
}

/*
 * Front end of a layer in a chain: the LN of Eq. 1 taken as RMS normalisation with unit gain,
 *   h_t = x_t / sqrt(mean_c(x_tc^2) + eps).
 * (The q/k/v projections that follow are plain products: dash_oracle_project.)
 */
int dash_oracle_rmsnorm(const double *x, int64_t m, int32_t d, double eps, double *out) {
    if (!x || !out || m < 0 || d <= 0 || eps < 0.0) return -1;
    for (int64_t i = 0; i < m; ++i) {
        double ss = 0.0;
        for (int32_t c = 0; c < d; ++c) ss += x[(size_t)i * d + c] * x[(size_t)i * d + c];
        const double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (int32_t c = 0; c < d; ++c) out[(size_t)i * d + c] = x[(size_t)i * d + c] * inv;
    }
    return 0;
}

/*
 * Rotary position embedding of the Qwen2.5 / Llama-3 backbones the paper evaluates (Sec. 4.1), in the
 * "rotate-half" pairing those models use: for a head vector u of row t, position p_t = pos[t] (the
 * token's ORIGINAL position: the compacted active sequence of Sec. 3.4 keeps the position ids) and
 * i < dh/2 with angle a = p_t * theta^(-2i/dh):
 *     out[i]        = u[i] cos a - u[i + dh/2] sin a
 *     out[i + dh/2] = u[i] sin a + u[i + dh/2] cos a.
 * u, out: [m, heads, dh]; dh even.
 */
int dash_oracle_rope(const double *u, const int32_t *pos, int64_t m, int32_t heads, int32_t dh, double theta,
                     double *out) {
    if (!u || !pos || !out || m < 0 || heads <= 0 || dh <= 0 || dh % 2 != 0 || !(theta > 0.0)) return -1;
    const int32_t half = dh / 2;
    for (int64_t t = 0; t < m; ++t)
        for (int32_t hd = 0; hd < heads; ++hd) {
            const double *ur = u + ((size_t)t * heads + hd) * dh;
            double *orow = out + ((size_t)t * heads + hd) * dh;
            for (int32_t i = 0; i < half; ++i) {
                const double a = (double)pos[t] * pow(theta, -2.0 * (double)i / (double)dh);
                const double c = cos(a), sn = sin(a);
                orow[i] = ur[i] * c - ur[i + half] * sn;
                orow[i + half] = ur[i] * sn + ur[i + half] * c;
            }
        }
    return 0;
}

/*
 * Second half of a block (Alg. 1 step 7): out = x + FFN(LN(x)), LN as in dash_oracle_rmsnorm, FFN the
 * gated feed-forward of the backbones the paper evaluates (Sec. 4.1):
 *     h = LN(x);  a = silu(h W_gate) * (h W_up);  out = x + a W_down,     silu(z) = z / (1 + exp(-z)).
 * x, out: [rows, d]; w_gate, w_up: [d, m]; w_down: [m, d].
 */
int dash_oracle_ffn_swiglu(const double *x, const double *w_gate, const double *w_up, const double *w_down,
                           int64_t rows, int32_t d, int32_t m, double eps, double *out) {
    if (!x || !w_gate || !w_up || !w_down || !out || rows < 0 || d <= 0 || m <= 0 || eps < 0.0) return -1;
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double *h = (double *)malloc(sizeof(double) * (size_t)d);
        double *a = (double *)malloc(sizeof(double) * (size_t)m);
        if (!h || !a) {
            rc = -2;
            free(h);
            free(a);
            continue;
        }
        const double *xr = x + (size_t)i * d;
        double ss = 0.0;
        for (int32_t c = 0; c < d; ++c) ss += xr[c] * xr[c];
        const double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (int32_t c = 0; c < d; ++c) h[c] = xr[c] * inv;
        for (int32_t f = 0; f < m; ++f) {
            double g = 0.0, u = 0.0;
            for (int32_t c = 0; c < d; ++c) {
                g += h[c] * w_gate[(size_t)c * m + f];
                u += h[c] * w_up[(size_t)c * m + f];
            }
            a[f] = g / (1.0 + exp(-g)) * u;
        }
        double *orow = out + (size_t)i * d;
        for (int32_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int32_t f = 0; f < m; ++f) acc += a[f] * w_down[(size_t)f * d + c];
            orow[c] = xr[c] + acc;
        }
        free(h);
        free(a);
    }
    return rc;
}

/*
 * Halted tokens keep the state they had when they halted (Sec. 3.4): rows[t] is written to
 * full[idx[t]] for every t with sel == NULL or sel[t] == sel_value. idx holds original positions in [0, N).
 */
int dash_oracle_scatter_rows(const double *rows, const int32_t *idx, const uint8_t *sel, int32_t sel_value,
                             int64_t n, int32_t d, int64_t N, double *full) {
    if (!rows || !idx || !full || n < 0 || d <= 0 || N < 0) return -1;
    for (int64_t t = 0; t < n; ++t) {
        if (sel && sel[t] != (uint8_t)sel_value) continue;
        if (idx[t] < 0 || idx[t] >= N) return -3;
        memcpy(full + (size_t)idx[t] * d, rows + (size_t)t * d, sizeof(double) * (size_t)d);
    }
    return 0;
}

/* H~ = H + U, element by element. */
int dash_oracle_residual(const double *x, const double *delta, int64_t m, int32_t d, double *x_next) {
    if (!x || !delta || !x_next || m < 0 || d <= 0) return -1;
    for (int64_t e = 0; e < m * (int64_t)d; ++e) x_next[e] = x[e] + delta[e];
    return 0;
}

/*
 * Per-token score. ABS: ||U_t||_2 (Eq. 2). REL: ||U_t||_2 / max(||H_t||_2, eps),
 * H_t being the residual-stream row that entered the block.
 */
int dash_oracle_scores(const double *delta, const double *x, int64_t m, int32_t d, int32_t kind,
                       double *scores) {
    if (!delta || !scores || m < 0 || d <= 0) return -1;
    if (kind != ORACLE_SCORE_REL && kind != ORACLE_SCORE_ABS) return -1;
    if (kind == ORACLE_SCORE_REL && !x) return -1;
    for (int64_t i = 0; i < m; ++i) {
        double sd = 0.0, sx = 0.0;
        for (int32_t c = 0; c < d; ++c) sd += delta[(size_t)i * d + c] * delta[(size_t)i * d + c];
        if (kind == ORACLE_SCORE_REL) {
            for (int32_t c = 0; c < d; ++c) sx += x[(size_t)i * d + c] * x[(size_t)i * d + c];
            double nx = sqrt(sx);
            if (nx < ORACLE_NORM_EPS) nx = ORACLE_NORM_EPS;
            scores[i] = sqrt(sd) / nx;
        } else {
            scores[i] = sqrt(sd);
        }
    }
    return 0;
}

static int row_is_protected(int64_t i, int64_t n, int64_t n_first, int64_t n_last) {
    return i < n_first || i >= n - n_last;
}

/*
 * Threshold form of the cut: halt row i iff score_i < tau and the row is not in
 * the protected prefix/suffix of the current active order. A score equal to tau,
 * or a NaN score, is kept.
 */
int dash_oracle_decide_threshold(const double *scores, int64_t n, double tau, int64_t n_first,
                                 int64_t n_last, uint8_t *halt) {
    if (!scores || !halt || n < 0 || n_first < 0 || n_last < 0) return -1;
    for (int64_t i = 0; i < n; ++i)
        halt[i] = (!row_is_protected(i, n, n_first, n_last) && scores[i] < tau) ? 1 : 0;
    return 0;
}

typedef struct {
    double s;
    int64_t i;
} scored_row;

/*
 * Order in which TopK ranks scores. Eq. 3 ranks real numbers; for the values a float can also hold the
 * reading taken is one total order
 *     -inf < ... < -0.0 = +0.0 < ... < +inf < NaN        (every NaN equal to every other NaN)
 * so that the selection is defined for any input: a NaN score ranks highest (the threshold form keeps NaN
 * rows too: "score < tau" is false for them), and the two zeros tie and are told apart by row like any tie.
 * Returns -1, 0 or 1.
 */
static int score_order(double a, double b) {
    const int an = isnan(a), bn = isnan(b);
    if (an || bn) return an - bn;
    return (a > b) - (a < b);
}

static int by_score_desc_then_row(const void *a, const void *b) {
    const scored_row *x = (const scored_row *)a, *y = (const scored_row *)b;
    const int c = score_order(x->s, y->s);
    if (c != 0) return -c;
    return (x->i > y->i) - (x->i < y->i);
}

/*
 * TopK form (Eq. 3): keep k_keep rows in total. Protected rows are always kept
 * and count towards k_keep; of the others, those with the highest scores are
 * kept (in the order of score_order: NaN above +inf, -0.0 equal to +0.0); among
 * equal scores the earlier row is kept first. If k_keep is not larger than the
 * number of protected rows, every unprotected row halts.
 */
int dash_oracle_decide_topk(const double *scores, int64_t n, int64_t k_keep, int64_t n_first,
                            int64_t n_last, uint8_t *halt) {
    if (!scores || !halt || n < 0 || k_keep < 0 || n_first < 0 || n_last < 0) return -1;
    scored_row *cand = (scored_row *)malloc((size_t)(n > 0 ? n : 1) * sizeof(scored_row));
    if (!cand) return -2;
    int64_t n_cand = 0, n_prot = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (row_is_protected(i, n, n_first, n_last)) {
            halt[i] = 0;
            ++n_prot;
        } else {
            halt[i] = 1;
            cand[n_cand].s = scores[i];
            cand[n_cand].i = i;
            ++n_cand;
        }
    }
    qsort(cand, (size_t)n_cand, sizeof(scored_row), by_score_desc_then_row);
    int64_t quota = k_keep - n_prot;
    if (quota < 0) quota = 0;
    if (quota > n_cand) quota = n_cand;
    for (int64_t c = 0; c < quota; ++c) halt[cand[c].i] = 0;
    free(cand);
    return 0;
}

static int by_score_asc_then_row(const void *a, const void *b) {
    const scored_row *x = (const scored_row *)a, *y = (const scored_row *)b;
    const int c = score_order(x->s, y->s);
    if (c != 0) return c;
    return (x->i > y->i) - (x->i < y->i);
}

/*
 * The direction control of the ablation (Sec. 5.4, "Directionality"): same budget, but the rows with the LOWEST
 * scores (lowest in the order of score_order, so NaN rows halt first) are kept, i.e. the high-Delta tokens halt.
 * Everything else as in dash_oracle_decide_topk. (Random
 * halting, the other control, is the ordinary TopK on scores drawn at random by the caller.)
 */
int dash_oracle_decide_topk_keep_low(const double *scores, int64_t n, int64_t k_keep, int64_t n_first,
                                     int64_t n_last, uint8_t *halt) {
    if (!scores || !halt || n < 0 || k_keep < 0 || n_first < 0 || n_last < 0) return -1;
    scored_row *cand = (scored_row *)malloc((size_t)(n > 0 ? n : 1) * sizeof(scored_row));
    if (!cand) return -2;
    int64_t n_cand = 0, n_prot = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (row_is_protected(i, n, n_first, n_last)) {
            halt[i] = 0;
            ++n_prot;
        } else {
            halt[i] = 1;
            cand[n_cand].s = scores[i];
            cand[n_cand].i = i;
            ++n_cand;
        }
    }
    qsort(cand, (size_t)n_cand, sizeof(scored_row), by_score_asc_then_row);
    int64_t quota = k_keep - n_prot;
    if (quota < 0) quota = 0;
    if (quota > n_cand) quota = n_cand;
    for (int64_t c = 0; c < quota; ++c) halt[cand[c].i] = 0;
    free(cand);
    return 0;
}

/*
 * Stable compaction: surviving rows in their original order.
 *   new_idx [<= n], x_compact [<= n, d] (may be NULL together with x_next), *n_out.
 */
int dash_oracle_compact(const uint8_t *halt, const int32_t *active_idx, const double *x_next,
                        int64_t n, int32_t d, int32_t *new_idx, double *x_compact, int64_t *n_out) {
    if (!halt || !active_idx || !new_idx || !n_out || n < 0) return -1;
    if ((x_next == NULL) != (x_compact == NULL)) return -1;
    int64_t p = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (halt[i]) continue;
        new_idx[p] = active_idx[i];
        if (x_next) memcpy(x_compact + (size_t)p * d, x_next + (size_t)i * d, (size_t)d * sizeof(double));
        ++p;
    }
    *n_out = p;
    return 0;
}

/*
 * Number of tokens kept out of n.
 *   paper_impl_rounding == 0 : K = floor((1 - rho) * n)                    (Eq. 3), as real arithmetic on
 *                              the decimal rho would give it (see the snap below)
 *   paper_impl_rounding != 0 : n - round(rho * (n - n_first - n_last))     (App. A, Table 5 caption)
 */
int64_t dash_oracle_keep_count(int64_t n, double rho, int64_t n_first, int64_t n_last,
                               int32_t paper_impl_rounding) {
    if (n < 0 || rho < 0.0 || rho >= 1.0 || n_first < 0 || n_last < 0) return -1;
    if (!paper_impl_rounding) {
        /* floor((1 - rho) n) = n - ceil(rho n) for integer n. rho is a decimal the caller wrote (0.4, 0.667) and
         * its double is not that decimal: a product that lands within 1e-9 (relative) of an integer is taken
         * to be that integer, so that rho = 0.667, n = 1000 drops 667 rows, not 668. */
        double dropped = rho * (double)n;
        const double nearest = nearbyint(dropped);
        if (fabs(dropped - nearest) <= 1e-9 * fmax(1.0, fabs(dropped))) dropped = nearest;
        return n - (int64_t)ceil(dropped);
    }
    const int64_t n_fix = n_first + n_last;
    if (n <= n_fix) return n;
    const int64_t drop = llround(rho * (double)(n - n_fix));
    return n - drop;
}

/* Per-layer FLOPs proxy A(n) = 4 n d^2 + 2 n^2 d + 2 n d m (App. A, Eq. 4). */
double dash_oracle_flops_A(double n, double d, double m) {
    return 4.0 * n * d * d + 2.0 * n * n * d + 2.0 * n * d * m;
}

/* C_full = L A(n); C_ours = l_s A(n) + (L - l_s) A(n_hat)   (App. A, Eq. 6-7). */
double dash_oracle_flops_full(double n, double d, double m, double L) {
    return L * dash_oracle_flops_A(n, d, m);
}

double dash_oracle_flops_single_shot(double n, double n_hat, double d, double m, double L, double l_s) {
    return l_s * dash_oracle_flops_A(n, d, m) + (L - l_s) * dash_oracle_flops_A(n_hat, d, m);
}
