/*
 * Driver for a sanitizer build of the CPU oracle (tests/test_sanitizers.py compiles this file together with
 * oracle/varlen_attn_oracle.c under -fsanitize=address,undefined and runs it).  Every buffer is allocated at
 * exactly the size the oracle's comments state, so that an index past an array's end is an error the
 * sanitizer reports; on top of that the row-subset entry points are compared with the full ones.
 * Exit status 0 and "ok" on success.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_varlen_attn_fwd(const float *, const float *, const float *, const int32_t *, int, int, int, int, int,
                           double, double *, double *);
int oracle_varlen_attn_fwd_rows(const float *, const float *, const float *, const int32_t *, int, int, int, int,
                                int, double, const int64_t *, int64_t, double *, double *);
int oracle_varlen_attn_bwd(const float *, const float *, const float *, const float *, const int32_t *, int, int,
                           int, int, int, double, double *, double *, double *);
int oracle_varlen_attn_bwd_saved_o(const float *, const float *, const float *, const float *, const double *,
                                   const int32_t *, int, int, int, int, int, double, double *, double *, double *);
int oracle_varlen_attn_bwd_q_rows(const float *, const float *, const float *, const float *, const double *,
                                  const int32_t *, int, int, int, int, int, double, const int64_t *, int64_t,
                                  double *);
int oracle_varlen_attn_bwd_kv_rows(const float *, const float *, const float *, const float *, const double *,
                                   const int32_t *, int, int, int, int, int, double, int, const int64_t *, int64_t,
                                   double *, double *);
int oracle_attn_merge(const float *, const double *, int, int, int, int, double *, double *);

static unsigned long long state = 88172645463325252ull;
static float rnd(void) {  /* xorshift, values in [-1, 1) on a 1/256 grid (exact in bf16) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((int)(state % 512) - 256) / 256.0f;
}
static float *fill(size_t n) {
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static double *dalloc(size_t n) { return (double *)calloc(n ? n : 1, sizeof(double)); }
static int fails = 0;
static void expect(int cond, const char *what) {
    if (!cond) { printf("FAILED: %s\n", what); ++fails; }
}
static double maxdiff(const double *a, const double *b, size_t n) {
    double m = 0;
    for (size_t i = 0; i < n; ++i) { double d = fabs(a[i] - b[i]); if (!(d <= m)) m = d; }
    return m;
}

int main(void) {
    /* ragged batch with an empty sample and a one-token sample; grouped query heads */
    const int32_t cu[] = {0, 5, 5, 6, 23, 40};
    const int B = 5, Hq = 4, Hkv = 2, D = 8, T = 40;
    const double scale = 0.35;
    float *q = fill((size_t)T * Hq * D), *k = fill((size_t)T * Hkv * D), *v = fill((size_t)T * Hkv * D);
    float *dout = fill((size_t)T * Hq * D);
    for (int causal = 0; causal < 2; ++causal) {
        double *o = dalloc((size_t)T * Hq * D), *lse = dalloc((size_t)Hq * T);
        expect(oracle_varlen_attn_fwd(q, k, v, cu, B, Hq, Hkv, D, causal, scale, o, lse) == 0, "fwd");
        int64_t rows[40];
        for (int i = 0; i < T; ++i) rows[i] = T - 1 - i;  /* every row, backwards */
        double *o_r = dalloc((size_t)T * Hq * D), *lse_r = dalloc((size_t)T * Hq);
        expect(oracle_varlen_attn_fwd_rows(q, k, v, cu, B, Hq, Hkv, D, causal, scale, rows, T, o_r, lse_r) == 0,
               "fwd_rows");
        double worst = 0;
        for (int i = 0; i < T; ++i)
            for (int h = 0; h < Hq; ++h) {
                double d = maxdiff(o_r + ((size_t)i * Hq + h) * D, o + ((size_t)rows[i] * Hq + h) * D, D);
                if (d > worst) worst = d;
                d = fabs(lse_r[i * Hq + h] - lse[(size_t)h * T + rows[i]]);
                if (d > worst) worst = d;
            }
        expect(worst == 0, "fwd_rows == fwd");

        double *dq = dalloc((size_t)T * Hq * D), *dk = dalloc((size_t)T * Hkv * D), *dv = dalloc((size_t)T * Hkv * D);
        expect(oracle_varlen_attn_bwd(q, k, v, dout, cu, B, Hq, Hkv, D, causal, scale, dq, dk, dv) == 0, "bwd");
        double *dq2 = dalloc((size_t)T * Hq * D), *dk2 = dalloc((size_t)T * Hkv * D), *dv2 = dalloc((size_t)T * Hkv * D);
        expect(oracle_varlen_attn_bwd_saved_o(q, k, v, dout, o, cu, B, Hq, Hkv, D, causal, scale, dq2, dk2, dv2) == 0,
               "bwd_saved_o");
        expect(maxdiff(dq, dq2, (size_t)T * Hq * D) < 1e-12 && maxdiff(dk, dk2, (size_t)T * Hkv * D) < 1e-12 &&
               maxdiff(dv, dv2, (size_t)T * Hkv * D) < 1e-12, "bwd_saved_o(own O) == bwd");
        double *dq_r = dalloc((size_t)T * Hq * D);
        expect(oracle_varlen_attn_bwd_q_rows(q, k, v, dout, NULL, cu, B, Hq, Hkv, D, causal, scale, rows, T, dq_r) == 0,
               "bwd_q_rows");
        worst = 0;
        for (int i = 0; i < T; ++i) {
            double d = maxdiff(dq_r + (size_t)i * Hq * D, dq + (size_t)rows[i] * Hq * D, (size_t)Hq * D);
            if (d > worst) worst = d;
        }
        expect(worst < 1e-12, "bwd_q_rows == bwd");
        for (int c = 0; c < Hkv; ++c) {
            double *dk_r = dalloc((size_t)T * D), *dv_r = dalloc((size_t)T * D);
            expect(oracle_varlen_attn_bwd_kv_rows(q, k, v, dout, o, cu, B, Hq, Hkv, D, causal, scale, c, rows, T, dk_r,
                                                  dv_r) == 0, "bwd_kv_rows");
            worst = 0;
            for (int i = 0; i < T; ++i) {
                double d = maxdiff(dk_r + (size_t)i * D, dk + ((size_t)rows[i] * Hkv + c) * D, D);
                if (d > worst) worst = d;
                d = maxdiff(dv_r + (size_t)i * D, dv + ((size_t)rows[i] * Hkv + c) * D, D);
                if (d > worst) worst = d;
            }
            expect(worst < 1e-12, "bwd_kv_rows == bwd");
            free(dk_r); free(dv_r);
        }
        /* rejected arguments return an error and touch nothing */
        expect(oracle_varlen_attn_fwd(q, k, v, cu, B, Hq, 3, D, causal, scale, o, lse) != 0, "Hq % Hkv != 0 rejected");
        rows[0] = T;
        expect(oracle_varlen_attn_fwd_rows(q, k, v, cu, B, Hq, Hkv, D, causal, scale, rows, T, o_r, lse_r) != 0,
               "row index past the end rejected");
        free(o); free(lse); free(o_r); free(lse_r); free(dq); free(dk); free(dv); free(dq2); free(dk2); free(dv2);
        free(dq_r);
    }
    /* merge of three parts, one of them empty for some rows */
    {
        const int P = 3, H = 2;
        float *op = fill((size_t)P * T * H * D);
        double *lp = dalloc((size_t)P * H * T);
        for (size_t i = 0; i < (size_t)P * H * T; ++i) lp[i] = (i % 7 == 0) ? -INFINITY : (double)rnd();
        double *o = dalloc((size_t)T * H * D), *lse = dalloc((size_t)H * T);
        expect(oracle_attn_merge(op, lp, P, T, H, D, o, lse) == 0, "merge");
        int finite = 1;
        for (size_t i = 0; i < (size_t)T * H * D; ++i) finite &= isfinite(o[i]) != 0;
        expect(finite, "merge output finite");
        free(op); free(lp); free(o); free(lse);
    }
    free(q); free(k); free(v); free(dout);
    if (fails) return 1;
    printf("ok\n");
    return 0;
}
