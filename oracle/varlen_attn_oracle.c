/*
 * CPU oracle for variable-length packed self-attention (forward and backward), fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  Only tests, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it; the product path never does.  It shares no code,
 * header or table with the HIP kernels.
 *
 * What it computes.  The paper (Section 6, "Efficient Operators") adopts an exact
 * tiled attention algorithm for its attention layers, so the result has a plain
 * definition: scaled-dot-product softmax attention.  Samples of a packed sequence
 * never attend to each other (Section 2.1, hybrid packing, Fig. 3c); encoder
 * attention is full inside a sample (Section 2.2, ViT tokens; Section 4.1.1 says
 * the Ulysses state keeps full attention per rank); LLM attention is causal
 * (Section 4.1.1, parallelism selection rationale).  The paper prints no formula,
 * so the textbook one is written out here:
 *
 *   for sample s, rows i, j in [cu[s], cu[s+1]), query head h, kv head c = h / (Hq/Hkv):
 *     allowed(i,j) = (not causal) or (j <= i)
 *     S_ij  = scale * sum_d Q[i,h,d] * K[j,c,d]
 *     LSE_i = ln sum_{j allowed} exp(S_ij)            (evaluated as max + ln sum exp(. - max))
 *     P_ij  = exp(S_ij - LSE_i)
 *     O[i,h,:] = sum_j P_ij * V[j,c,:]
 *   backward, given dO:
 *     Delta_i   = sum_d dO[i,h,d] * O[i,h,d]
 *     dP_ij     = sum_d dO[i,h,d] * V[j,c,d]
 *     dS_ij     = P_ij * (dP_ij - Delta_i)
 *     dQ[i,h,:] = scale * sum_j dS_ij * K[j,c,:]
 *     dK[j,c,:] = scale * sum_{h in group c} sum_i dS_ij * Q[i,h,:]
 *     dV[j,c,:] = sum_{h in group c} sum_i P_ij * dO[i,h,:]
 *
 * Layouts: Q, O, dO, dQ are [T, Hq, D]; K, V, dK, dV are [T, Hkv, D]; LSE is [Hq, T];
 * all row-major.  Inputs are float (every bf16 value is exactly a float), all
 * arithmetic and all outputs are double.  No blocking, no fusion, no online softmax.
 *
 * Pins (tests/test_oracle_pins.py): brute force without max-subtraction, Q = 0
 * closed forms, length-1 sequences, packed == alone, permutation and shift
 * invariances, causal row == non-causal prefix, GQA == repeated-head MHA, central
 * finite differences, dense autograd of a library softmax, row identities, and
 * large-logit stability against extended precision; the stored-O variant against its
 * first-order closed form, the row-subset variants against the full backward.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int check_args(const int32_t *cu, int B, int Hq, int Hkv, int D) {
    if (B < 0 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0 || !cu) return ORACLE_BAD_ARG;
    if (cu[0] != 0) return ORACLE_BAD_ARG;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] < cu[s]) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

/* index of the sample that holds packed row t (samples of length 0 hold no row) */
static int sample_of_row(const int32_t *cu, int B, int64_t t) {
    for (int s = 0; s < B; ++s)
        if (t >= cu[s] && t < cu[s + 1]) return s;
    return -1;
}

/*
 * One output row: scores of query (i,h) against keys j in [j0, j1), then LSE, then O.
 * `score` is scratch of at least j1 - j0 doubles.  Returns LSE; writes D doubles to o_row.
 */
static double attend_row(const float *q, const float *k, const float *v, int Hq, int Hkv, int D,
                         double scale, int64_t i, int h, int64_t j0, int64_t j1,
                         double *score, double *o_row) {
    const int c = h / (Hq / Hkv);
    const float *qi = q + ((size_t)i * Hq + h) * D;
    double m = -INFINITY;
    for (int64_t j = j0; j < j1; ++j) {
        const float *kj = k + ((size_t)j * Hkv + c) * D;
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)qi[d] * (double)kj[d];
        score[j - j0] = scale * acc;
        if (score[j - j0] > m) m = score[j - j0];
    }
    double sum = 0.0;
    for (int64_t j = j0; j < j1; ++j) sum += exp(score[j - j0] - m);
    const double lse = m + log(sum);
    for (int d = 0; d < D; ++d) o_row[d] = 0.0;
    for (int64_t j = j0; j < j1; ++j) {
        const double p = exp(score[j - j0] - lse);
        const float *vj = v + ((size_t)j * Hkv + c) * D;
        for (int d = 0; d < D; ++d) o_row[d] += p * (double)vj[d];
    }
    return lse;
}

/*
 * Forward for a list of packed rows (all query heads of each listed row).
 *   rows[n_rows]  : packed row indices in [0, T)
 *   o_rows        : [n_rows, Hq, D] double
 *   lse_rows      : [n_rows, Hq]    double
 * Each output row depends only on its own sample's K and V, so a subset of rows is exact.
 */
int oracle_varlen_attn_fwd_rows(const float *q, const float *k, const float *v, const int32_t *cu,
                                int B, int Hq, int Hkv, int D, int causal, double scale,
                                const int64_t *rows, int64_t n_rows, double *o_rows,
                                double *lse_rows) {
    int rc = check_args(cu, B, Hq, Hkv, D);
    if (rc) return rc;
    int64_t max_len = 0;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] - cu[s] > max_len) max_len = cu[s + 1] - cu[s];
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= cu[B]) return ORACLE_BAD_ARG;
    int failed = 0;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        if (!score) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int64_t r = 0; r < n_rows; ++r) {
            for (int h = 0; h < Hq; ++h) {
                if (!score) continue;
                const int64_t i = rows[r];
                const int s = sample_of_row(cu, B, i);
                const int64_t j0 = cu[s];
                const int64_t j1 = causal ? i + 1 : cu[s + 1];
                lse_rows[r * Hq + h] = attend_row(q, k, v, Hq, Hkv, D, scale, i, h, j0, j1, score,
                                                  o_rows + ((size_t)r * Hq + h) * D);
            }
        }
        free(score);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/* Forward for every row.  o: [T, Hq, D] double, lse: [Hq, T] double. */
int oracle_varlen_attn_fwd(const float *q, const float *k, const float *v, const int32_t *cu, int B,
                           int Hq, int Hkv, int D, int causal, double scale, double *o,
                           double *lse) {
    int rc = check_args(cu, B, Hq, Hkv, D);
    if (rc) return rc;
    const int64_t T = cu[B];
    int64_t max_len = 0;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] - cu[s] > max_len) max_len = cu[s + 1] - cu[s];
    int failed = 0;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        if (!score) {
#pragma omp atomic write
            failed = 1;
        }
        for (int s = 0; s < B; ++s) {
#pragma omp for collapse(2) schedule(dynamic, 4) nowait
            for (int64_t i = cu[s]; i < cu[s + 1]; ++i) {
                for (int h = 0; h < Hq; ++h) {
                    if (!score) continue;
                    const int64_t j1 = causal ? i + 1 : cu[s + 1];
                    lse[(size_t)h * T + i] = attend_row(q, k, v, Hq, Hkv, D, scale, i, h, cu[s], j1,
                                                        score, o + ((size_t)i * Hq + h) * D);
                }
            }
        }
        free(score);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/*
 * Backward for every row.  dq: [T, Hq, D], dk, dv: [T, Hkv, D], all double, fully
 * overwritten.  P and LSE are the oracle's own fp64 values (recomputed here), not
 * anything a caller saved.  Delta_i = <dO_i, O_i> uses the oracle's own fp64 O when
 * o_saved is NULL (the definition), else the rows of o_saved: double [T, Hq, D], the
 * forward output as a caller stored it (a training framework saves O in bf16 and the
 * backward interface reads it back; this variant states what the exact gradient
 * arithmetic gives from that stored O, so that the cost of the interface and the error
 * of an implementation can be told apart).  Two sweeps so that every output row has one
 * writer:
 *   sweep 1, per query row (i,h): LSE_i, O_i, Delta_i, dQ_i
 *   sweep 2, per key row (j,c):   dK_j, dV_j from LSE and Delta of sweep 1
 */
static int bwd_impl(const float *q, const float *k, const float *v, const float *dout,
                    const double *o_saved, const int32_t *cu, int B, int Hq, int Hkv, int D,
                    int causal, double scale, double *dq, double *dk, double *dv) {
    int rc = check_args(cu, B, Hq, Hkv, D);
    if (rc) return rc;
    const int64_t T = cu[B];
    const int g = Hq / Hkv;
    int64_t max_len = 0;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] - cu[s] > max_len) max_len = cu[s + 1] - cu[s];
    double *lse = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * Hq);
    double *delta = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * Hq);
    if (!lse || !delta) {
        free(lse);
        free(delta);
        return ORACLE_NO_MEM;
    }
    int failed = 0;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        double *o_row = (double *)malloc(sizeof(double) * (size_t)D);
        if (!score || !o_row) {
#pragma omp atomic write
            failed = 1;
        }
        /* sweep 1 */
        for (int s = 0; s < B; ++s) {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int64_t i = cu[s]; i < cu[s + 1]; ++i) {
                for (int h = 0; h < Hq; ++h) {
                    if (!score || !o_row) continue;
                    const int c = h / g;
                    const int64_t j0 = cu[s];
                    const int64_t j1 = causal ? i + 1 : cu[s + 1];
                    const double l = attend_row(q, k, v, Hq, Hkv, D, scale, i, h, j0, j1, score, o_row);
                    const float *doi = dout + ((size_t)i * Hq + h) * D;
                    const double *oi = o_saved ? o_saved + ((size_t)i * Hq + h) * D : o_row;
                    double dl = 0.0;
                    for (int d = 0; d < D; ++d) dl += (double)doi[d] * oi[d];
                    lse[(size_t)h * T + i] = l;
                    delta[(size_t)h * T + i] = dl;
                    double *dqi = dq + ((size_t)i * Hq + h) * D;
                    for (int d = 0; d < D; ++d) dqi[d] = 0.0;
                    for (int64_t j = j0; j < j1; ++j) {
                        const float *kj = k + ((size_t)j * Hkv + c) * D;
                        const float *vj = v + ((size_t)j * Hkv + c) * D;
                        const double p = exp(score[j - j0] - l);
                        double dp = 0.0;
                        for (int d = 0; d < D; ++d) dp += (double)doi[d] * (double)vj[d];
                        const double ds = p * (dp - dl);
                        for (int d = 0; d < D; ++d) dqi[d] += ds * (double)kj[d];
                    }
                    for (int d = 0; d < D; ++d) dqi[d] *= scale;
                }
            }
        }
        /* sweep 2 (the implicit barrier of the last omp-for above orders it after sweep 1) */
        for (int s = 0; s < B; ++s) {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int64_t j = cu[s]; j < cu[s + 1]; ++j) {
                for (int c = 0; c < Hkv; ++c) {
                    const float *kj = k + ((size_t)j * Hkv + c) * D;
                    const float *vj = v + ((size_t)j * Hkv + c) * D;
                    double *dkj = dk + ((size_t)j * Hkv + c) * D;
                    double *dvj = dv + ((size_t)j * Hkv + c) * D;
                    for (int d = 0; d < D; ++d) dkj[d] = dvj[d] = 0.0;
                    const int64_t i0 = causal ? j : cu[s];
                    for (int h = c * g; h < (c + 1) * g; ++h) {
                        for (int64_t i = i0; i < cu[s + 1]; ++i) {
                            const float *qi = q + ((size_t)i * Hq + h) * D;
                            const float *doi = dout + ((size_t)i * Hq + h) * D;
                            double sc = 0.0, dp = 0.0;
                            for (int d = 0; d < D; ++d) sc += (double)qi[d] * (double)kj[d];
                            for (int d = 0; d < D; ++d) dp += (double)doi[d] * (double)vj[d];
                            const double p = exp(scale * sc - lse[(size_t)h * T + i]);
                            const double ds = p * (dp - delta[(size_t)h * T + i]);
                            for (int d = 0; d < D; ++d) dvj[d] += p * (double)doi[d];
                            for (int d = 0; d < D; ++d) dkj[d] += ds * (double)qi[d];
                        }
                    }
                    for (int d = 0; d < D; ++d) dkj[d] *= scale;
                }
            }
        }
        free(score);
        free(o_row);
    }
    free(lse);
    free(delta);
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

int oracle_varlen_attn_bwd(const float *q, const float *k, const float *v, const float *dout,
                           const int32_t *cu, int B, int Hq, int Hkv, int D, int causal,
                           double scale, double *dq, double *dk, double *dv) {
    return bwd_impl(q, k, v, dout, NULL, cu, B, Hq, Hkv, D, causal, scale, dq, dk, dv);
}

/* The same with Delta formed from a stored forward output o_saved (double [T, Hq, D]). */
int oracle_varlen_attn_bwd_saved_o(const float *q, const float *k, const float *v,
                                   const float *dout, const double *o_saved, const int32_t *cu,
                                   int B, int Hq, int Hkv, int D, int causal, double scale,
                                   double *dq, double *dk, double *dv) {
    if (!o_saved) return ORACLE_BAD_ARG;
    return bwd_impl(q, k, v, dout, o_saved, cu, B, Hq, Hkv, D, causal, scale, dq, dk, dv);
}

/*
 * dQ for a list of packed query rows (all query heads of each listed row).  Given K and V, dQ_i
 * depends on no other query row, so a subset of rows is exact at any sample length:
 *     dQ[i,h,:] = scale * sum_j P_ij (dP_ij - Delta_i) K[j,c,:].
 *   rows[n_rows] : packed row indices;  dq_rows : [n_rows, Hq, D] double
 *   o_saved      : NULL (Delta from the oracle's own O) or double [T, Hq, D] (see bwd_impl)
 */
int oracle_varlen_attn_bwd_q_rows(const float *q, const float *k, const float *v,
                                  const float *dout, const double *o_saved, const int32_t *cu,
                                  int B, int Hq, int Hkv, int D, int causal, double scale,
                                  const int64_t *rows, int64_t n_rows, double *dq_rows) {
    int rc = check_args(cu, B, Hq, Hkv, D);
    if (rc) return rc;
    const int g = Hq / Hkv;
    int64_t max_len = 0;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] - cu[s] > max_len) max_len = cu[s + 1] - cu[s];
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= cu[B]) return ORACLE_BAD_ARG;
    int failed = 0;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        double *o_row = (double *)malloc(sizeof(double) * (size_t)D);
        if (!score || !o_row) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            for (int h = 0; h < Hq; ++h) {
                if (!score || !o_row) continue;
                const int64_t i = rows[r];
                const int s = sample_of_row(cu, B, i);
                const int c = h / g;
                const int64_t j0 = cu[s];
                const int64_t j1 = causal ? i + 1 : cu[s + 1];
                const double l = attend_row(q, k, v, Hq, Hkv, D, scale, i, h, j0, j1, score, o_row);
                const float *doi = dout + ((size_t)i * Hq + h) * D;
                const double *oi = o_saved ? o_saved + ((size_t)i * Hq + h) * D : o_row;
                double dl = 0.0;
                for (int d = 0; d < D; ++d) dl += (double)doi[d] * oi[d];
                double *dqi = dq_rows + ((size_t)r * Hq + h) * D;
                for (int d = 0; d < D; ++d) dqi[d] = 0.0;
                for (int64_t j = j0; j < j1; ++j) {
                    const float *kj = k + ((size_t)j * Hkv + c) * D;
                    const float *vj = v + ((size_t)j * Hkv + c) * D;
                    const double p = exp(score[j - j0] - l);
                    double dp = 0.0;
                    for (int d = 0; d < D; ++d) dp += (double)doi[d] * (double)vj[d];
                    const double ds = p * (dp - dl);
                    for (int d = 0; d < D; ++d) dqi[d] += ds * (double)kj[d];
                }
                for (int d = 0; d < D; ++d) dqi[d] *= scale;
            }
        }
        free(score);
        free(o_row);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/*
 * dK and dV for a list of packed key rows of ONE kv head c.  A key row's gradients sum over every
 * query row of its sample (and the query heads of group c), so LSE and Delta of all those query rows
 * are evaluated first (sweep 1, restricted to the samples that hold a listed row and to the heads of
 * the group), then the listed key rows (sweep 2):
 *     dV[j,c,:] = sum_{h in group c} sum_i P_ij dO[i,h,:]
 *     dK[j,c,:] = scale * sum_{h in group c} sum_i P_ij (dP_ij - Delta_i) Q[i,h,:]
 *   rows[n_rows] : packed row indices;  dk_rows, dv_rows : [n_rows, D] double
 *   o_saved      : NULL or double [T, Hq, D] (see bwd_impl)
 */
int oracle_varlen_attn_bwd_kv_rows(const float *q, const float *k, const float *v,
                                   const float *dout, const double *o_saved, const int32_t *cu,
                                   int B, int Hq, int Hkv, int D, int causal, double scale, int c,
                                   const int64_t *rows, int64_t n_rows, double *dk_rows,
                                   double *dv_rows) {
    int rc = check_args(cu, B, Hq, Hkv, D);
    if (rc) return rc;
    if (c < 0 || c >= Hkv) return ORACLE_BAD_ARG;
    const int64_t T = cu[B];
    const int g = Hq / Hkv;
    int64_t max_len = 0;
    for (int s = 0; s < B; ++s)
        if (cu[s + 1] - cu[s] > max_len) max_len = cu[s + 1] - cu[s];
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= T) return ORACLE_BAD_ARG;
    char *wanted = (char *)calloc((size_t)(B > 0 ? B : 1), 1); /* samples that hold a listed row */
    double *lse = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * g);
    double *delta = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * g);
    if (!wanted || !lse || !delta) {
        free(wanted);
        free(lse);
        free(delta);
        return ORACLE_NO_MEM;
    }
    for (int64_t r = 0; r < n_rows; ++r) wanted[sample_of_row(cu, B, rows[r])] = 1;
    int failed = 0;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        double *o_row = (double *)malloc(sizeof(double) * (size_t)D);
        if (!score || !o_row) {
#pragma omp atomic write
            failed = 1;
        }
        /* sweep 1: LSE and Delta, stored as [member of the group][row] */
        for (int s = 0; s < B; ++s) {
            if (!wanted[s]) continue;
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int64_t i = cu[s]; i < cu[s + 1]; ++i) {
                for (int m = 0; m < g; ++m) {
                    if (!score || !o_row) continue;
                    const int h = c * g + m;
                    const int64_t j1 = causal ? i + 1 : cu[s + 1];
                    const double l = attend_row(q, k, v, Hq, Hkv, D, scale, i, h, cu[s], j1, score, o_row);
                    const float *doi = dout + ((size_t)i * Hq + h) * D;
                    const double *oi = o_saved ? o_saved + ((size_t)i * Hq + h) * D : o_row;
                    double dl = 0.0;
                    for (int d = 0; d < D; ++d) dl += (double)doi[d] * oi[d];
                    lse[(size_t)m * T + i] = l;
                    delta[(size_t)m * T + i] = dl;
                }
            }
        }
        /* sweep 2: the listed key rows */
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t j = rows[r];
            const int s = sample_of_row(cu, B, j);
            const float *kj = k + ((size_t)j * Hkv + c) * D;
            const float *vj = v + ((size_t)j * Hkv + c) * D;
            double *dkj = dk_rows + (size_t)r * D;
            double *dvj = dv_rows + (size_t)r * D;
            for (int d = 0; d < D; ++d) dkj[d] = dvj[d] = 0.0;
            const int64_t i0 = causal ? j : cu[s];
            for (int m = 0; m < g; ++m) {
                const int h = c * g + m;
                for (int64_t i = i0; i < cu[s + 1]; ++i) {
                    const float *qi = q + ((size_t)i * Hq + h) * D;
                    const float *doi = dout + ((size_t)i * Hq + h) * D;
                    double sc = 0.0, dp = 0.0;
                    for (int d = 0; d < D; ++d) sc += (double)qi[d] * (double)kj[d];
                    for (int d = 0; d < D; ++d) dp += (double)doi[d] * (double)vj[d];
                    const double p = exp(scale * sc - lse[(size_t)m * T + i]);
                    const double ds = p * (dp - delta[(size_t)m * T + i]);
                    for (int d = 0; d < D; ++d) dvj[d] += p * (double)doi[d];
                    for (int d = 0; d < D; ++d) dkj[d] += ds * (double)qi[d];
                }
            }
            for (int d = 0; d < D; ++d) dkj[d] *= scale;
        }
        free(score);
        free(o_row);
    }
    free(wanted);
    free(lse);
    free(delta);
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/*
 * Merge of partial attention results over disjoint key/value shards.
 *
 * Where the paper needs it: context parallelism for overlong contexts (Section 4.1.2, 5D parallelism
 * for the LLM; Section 5.2, adaptive sample sharding) leaves every rank with the attention
 * of its queries over ONE shard of the keys; the full result is their combination.  The paper does
 * not print it; it follows from the definition.  With part p holding, for one (query row, head),
 *     O_p = sum_{j in shard p} exp(S_j - LSE_p) V_j,   LSE_p = ln sum_{j in shard p} exp(S_j)
 * the result over the union of the shards is
 *     LSE = ln sum_p exp(LSE_p),   O = sum_p exp(LSE_p - LSE) O_p.
 * A part whose shard held no key for this row has LSE_p = -infinity and weight 0 (its O_p is not
 * looked at); if every part is empty, O = 0 and LSE = -infinity.
 *
 * o_parts: float [P, T, H, D], lse_parts: double [P, H, T]; out o: double [T, H, D], lse: double [H, T].
 */
int oracle_attn_merge(const float *o_parts, const double *lse_parts, int P, int T, int H, int D,
                      double *o, double *lse) {
    if (P < 1 || T < 0 || H < 1 || D < 1 || !o_parts || !lse_parts || !o || !lse) return ORACLE_BAD_ARG;
    for (int i = 0; i < T; ++i)
        for (int h = 0; h < H; ++h) {
            double mx = -INFINITY;
            for (int p = 0; p < P; ++p) {
                double x = lse_parts[((size_t)p * H + h) * T + i];
                if (x > mx) mx = x;
            }
            double *orow = o + ((size_t)i * H + h) * D;
            for (int d = 0; d < D; ++d) orow[d] = 0.0;
            if (mx == -INFINITY) {
                lse[(size_t)h * T + i] = -INFINITY;
                continue;
            }
            double den = 0.0;
            for (int p = 0; p < P; ++p) den += exp(lse_parts[((size_t)p * H + h) * T + i] - mx);
            const double total = mx + log(den);
            lse[(size_t)h * T + i] = total;
            for (int p = 0; p < P; ++p) {
                const double x = lse_parts[((size_t)p * H + h) * T + i];
                if (x == -INFINITY) continue;
                const double wgt = exp(x - total);
                const float *prow = o_parts + (((size_t)p * T + i) * H + h) * D;
                for (int d = 0; d < D; ++d) orow[d] += wgt * (double)prow[d];
            }
        }
    return ORACLE_OK;
}
