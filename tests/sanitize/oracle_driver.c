/*
 * Driver for a sanitizer build of the CPU oracle (test infrastructure): reads small inputs from a file written by
 * the test, calls every oracle function once and writes all results to another file. Built by the test with
 * gcc -fsanitize=address,undefined together with oracle/dash_oracle.c; a bad access or undefined operation in the
 * oracle aborts the run, and the test also compares the results with those of the ordinary build.
 *
 * Input file : int64 header {n, Hq, Hkv, dh, d, m, N, k_keep, n_first, n_last, n_rows}, then doubles
 *              x[n,d] q[n,Hq,dh] k[n,Hkv,dh] v[n,Hkv,dh] w_o[Hq*dh,d] w_gate[d,m] w_up[d,m] w_down[m,d] tau theta,
 *              then int32 pos[n], then int64 rows[n_rows].
 * Output file: doubles, in the order written below.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int dash_oracle_attention_rows(const double *, const double *, const double *, const int32_t *, int64_t, int32_t,
                               int32_t, int32_t, int32_t, double, const int64_t *, int64_t, double *);
int dash_oracle_project(const double *, const double *, int64_t, int32_t, int32_t, double *);
int dash_oracle_rmsnorm(const double *, int64_t, int32_t, double, double *);
int dash_oracle_rope(const double *, const int32_t *, int64_t, int32_t, int32_t, double, double *);
int dash_oracle_ffn_swiglu(const double *, const double *, const double *, const double *, int64_t, int32_t, int32_t,
                           double, double *);
int dash_oracle_scatter_rows(const double *, const int32_t *, const uint8_t *, int32_t, int64_t, int32_t, int64_t,
                             double *);
int dash_oracle_residual(const double *, const double *, int64_t, int32_t, double *);
int dash_oracle_scores(const double *, const double *, int64_t, int32_t, int32_t, double *);
int dash_oracle_decide_threshold(const double *, int64_t, double, int64_t, int64_t, uint8_t *);
int dash_oracle_decide_topk(const double *, int64_t, int64_t, int64_t, int64_t, uint8_t *);
int dash_oracle_decide_topk_keep_low(const double *, int64_t, int64_t, int64_t, int64_t, uint8_t *);
int dash_oracle_compact(const uint8_t *, const int32_t *, const double *, int64_t, int32_t, int32_t *, double *,
                        int64_t *);
int64_t dash_oracle_keep_count(int64_t, double, int64_t, int64_t, int32_t);
double dash_oracle_flops_A(double, double, double);
double dash_oracle_flops_full(double, double, double, double);
double dash_oracle_flops_single_shot(double, double, double, double, double, double);

static void *xmalloc(size_t bytes) {
    void *p = malloc(bytes ? bytes : 1);
    if (!p) exit(3);
    return p;
}
static double *rd(FILE *f, size_t count) {
    double *p = (double *)xmalloc(count * sizeof(double));
    if (fread(p, sizeof(double), count, f) != count) exit(4);
    return p;
}
static void wr(FILE *f, const double *p, size_t count) {
    if (fwrite(p, sizeof(double), count, f) != count) exit(5);
}
static void wr_u8(FILE *f, const uint8_t *p, size_t count) {
    for (size_t i = 0; i < count; ++i) {
        const double v = p[i];
        wr(f, &v, 1);
    }
}
#define CHECK(call)            \
    do {                       \
        if ((call) != 0) {     \
            fprintf(stderr, "failed: %s\n", #call); \
            return 6;          \
        }                      \
    } while (0)

int main(int argc, char **argv) {
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int64_t h[11];
    if (fread(h, sizeof(int64_t), 11, in) != 11) return 4;
    const int64_t n = h[0], N = h[6], k_keep = h[7], n_first = h[8], n_last = h[9], n_rows = h[10];
    const int32_t Hq = (int32_t)h[1], Hkv = (int32_t)h[2], dh = (int32_t)h[3], d = (int32_t)h[4], m = (int32_t)h[5];
    const int32_t Da = Hq * dh;
    double *x = rd(in, (size_t)n * d), *q = rd(in, (size_t)n * Hq * dh), *k = rd(in, (size_t)n * Hkv * dh);
    double *v = rd(in, (size_t)n * Hkv * dh), *w_o = rd(in, (size_t)Da * d), *w_gate = rd(in, (size_t)d * m);
    double *w_up = rd(in, (size_t)d * m), *w_down = rd(in, (size_t)m * d), *tau = rd(in, 1), *theta = rd(in, 1);
    int32_t *pos = (int32_t *)xmalloc((size_t)n * sizeof(int32_t));
    int64_t *rows = (int64_t *)xmalloc((size_t)n_rows * sizeof(int64_t));
    if (fread(pos, sizeof(int32_t), (size_t)n, in) != (size_t)n) return 4;
    if (fread(rows, sizeof(int64_t), (size_t)n_rows, in) != (size_t)n_rows) return 4;

    int64_t *all = (int64_t *)xmalloc((size_t)n * sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i) all[i] = i;
    double *O = (double *)xmalloc((size_t)n * Da * sizeof(double));
    double *Osub = (double *)xmalloc((size_t)n_rows * Da * sizeof(double));
    double *delta = (double *)xmalloc((size_t)n * d * sizeof(double)), *xn = (double *)xmalloc((size_t)n * d * sizeof(double));
    double *s_rel = (double *)xmalloc((size_t)n * sizeof(double)), *s_abs = (double *)xmalloc((size_t)n * sizeof(double));
    uint8_t *halt = (uint8_t *)xmalloc((size_t)n);
    int32_t *new_idx = (int32_t *)xmalloc((size_t)n * sizeof(int32_t));
    double *xc = (double *)xmalloc((size_t)n * d * sizeof(double));
    double *tmp = (double *)xmalloc((size_t)n * (Hq * dh > d ? Hq * dh : d) * sizeof(double));
    double *full = (double *)xmalloc((size_t)N * d * sizeof(double));

    CHECK(dash_oracle_attention_rows(q, k, v, pos, n, Hq, Hkv, dh, 1, 0.3, all, n, O));
    wr(out, O, (size_t)n * Da);
    CHECK(dash_oracle_attention_rows(q, k, v, pos, n, Hq, Hkv, dh, 0, 0.3, rows, n_rows, Osub));
    wr(out, Osub, (size_t)n_rows * Da);
    CHECK(dash_oracle_project(O, w_o, n, Da, d, delta));
    wr(out, delta, (size_t)n * d);
    CHECK(dash_oracle_residual(x, delta, n, d, xn));
    wr(out, xn, (size_t)n * d);
    CHECK(dash_oracle_scores(delta, x, n, d, 0, s_rel));
    CHECK(dash_oracle_scores(delta, NULL, n, d, 1, s_abs));
    wr(out, s_rel, (size_t)n);
    wr(out, s_abs, (size_t)n);
    CHECK(dash_oracle_decide_threshold(s_rel, n, tau[0], n_first, n_last, halt));
    wr_u8(out, halt, (size_t)n);
    CHECK(dash_oracle_decide_topk_keep_low(s_rel, n, k_keep, n_first, n_last, halt));
    wr_u8(out, halt, (size_t)n);
    CHECK(dash_oracle_decide_topk(s_rel, n, k_keep, n_first, n_last, halt));
    wr_u8(out, halt, (size_t)n);
    int64_t n_out = 0;
    CHECK(dash_oracle_compact(halt, pos, xn, n, d, new_idx, xc, &n_out));
    {
        const double c = (double)n_out;
        wr(out, &c, 1);
        for (int64_t i = 0; i < n_out; ++i) {
            const double p = new_idx[i];
            wr(out, &p, 1);
        }
        wr(out, xc, (size_t)n_out * d);
    }
    CHECK(dash_oracle_rmsnorm(x, n, d, 1e-6, tmp));
    wr(out, tmp, (size_t)n * d);
    CHECK(dash_oracle_rope(q, pos, n, Hq, dh, theta[0], tmp));
    wr(out, tmp, (size_t)n * Hq * dh);
    CHECK(dash_oracle_ffn_swiglu(x, w_gate, w_up, w_down, n, d, m, 1e-6, tmp));
    wr(out, tmp, (size_t)n * d);
    for (int64_t i = 0; i < N * d; ++i) full[i] = -1.0;
    CHECK(dash_oracle_scatter_rows(xn, pos, halt, 1, n, d, N, full));
    wr(out, full, (size_t)N * d);
    {
        const double kc[4] = {(double)dash_oracle_keep_count(n, 0.667, 0, 0, 0),
                              (double)dash_oracle_keep_count(32768, 0.667, 64, 32, 1),
                              (double)dash_oracle_keep_count(n, 1.0, 0, 0, 0), dash_oracle_flops_A(8192, 3584, 18944)};
        wr(out, kc, 4);
        const double fl[2] = {dash_oracle_flops_full(8192, 3584, 18944, 28),
                              dash_oracle_flops_single_shot(8192, 2792, 3584, 18944, 28, 11)};
        wr(out, fl, 2);
    }
    /* invalid arguments must be refused, not dereferenced */
    if (dash_oracle_attention_rows(NULL, k, v, pos, n, Hq, Hkv, dh, 1, 0.3, all, n, O) == 0) return 7;
    if (dash_oracle_decide_topk(s_rel, -1, 1, 0, 0, halt) == 0) return 7;
    {
        int64_t bad_row = n;
        if (dash_oracle_attention_rows(q, k, v, pos, n, Hq, Hkv, dh, 1, 0.3, &bad_row, 1, O) == 0) return 7;
    }
    free(x); free(q); free(k); free(v); free(w_o); free(w_gate); free(w_up); free(w_down); free(tau); free(theta);
    free(pos); free(rows); free(all); free(O); free(Osub); free(delta); free(xn); free(s_rel); free(s_abs); free(halt);
    free(new_idx); free(xc); free(tmp); free(full);
    fclose(in);
    if (fclose(out) != 0) return 5;
    return 0;
}
