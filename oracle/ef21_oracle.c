/*
 * EF21 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded implementation of what the GPU hot path
 * computes, written from the paper (Richtarik, Sokolov, Fatkhullin, "EF21",
 * arXiv 2106.05203).  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * Precision.  All arithmetic is fp64.  State vectors (x, g_i, g), gradients and
 * compressor messages live in double arrays.  When `storage_f32` is non-zero every
 * value stored into such an array is first rounded to the nearest fp32, and the
 * difference that feeds Top-k is one fp32 subtraction, so that the selection is
 * decided in the same precision as on the GPU.  With `storage_f32 == 0` nothing is
 * rounded (pure fp64; used to measure fp32 drift and for exact identities).
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned against
 * something other than itself -- exhaustive subset search for Top-k, closed forms and
 * finite differences for the objective, k = d <=> gradient descent, the invariant
 * g = mean g_i, the one-step distortion bound and Theorem 1's rate for the
 * iteration.  The values f(x^t) of a full trajectory are "parity unpinned": the paper
 * prints no number for any run.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double store(double v, int storage_f32) { return storage_f32 ? (double)(float)v : v; }

/* ------------------------------------------------------------------------------------
 * Top-k compressor (Section 2.1: keep the k entries that are largest in absolute value,
 * zero the rest; alpha = k/d, Appendix F.2).
 *
 * Plain definition written out: order all d positions by |v_j| descending with a STABLE
 * sort, so that positions of equal magnitude stay in ascending index order (the paper
 * does not say how ties are broken; the reading taken here is "lower index wins", and +a
 * ties with -a, +0 with -0).  The first k positions of that order are kept.  They are
 * reported in ascending index order together with their (signed) values.
 * ------------------------------------------------------------------------------------ */
static void merge_runs(const double *mag, const int64_t *src, int64_t *dst, int64_t lo, int64_t mid,
                       int64_t hi) {
    int64_t a = lo, b = mid, o = lo;
    while (a < mid && b < hi) {
        /* take from the right run only when it is strictly larger: keeps the sort stable */
        if (mag[src[b]] > mag[src[a]]) dst[o++] = src[b++];
        else dst[o++] = src[a++];
    }
    while (a < mid) dst[o++] = src[a++];
    while (b < hi) dst[o++] = src[b++];
}

static int cmp_i64(const void *p, const void *q) {
    int64_t a = *(const int64_t *)p, b = *(const int64_t *)q;
    return (a > b) - (a < b);
}

/* returns 0 on success, -1 on bad arguments or allocation failure */
int ef21o_topk(const double *v, int64_t d, int64_t k, int32_t *out_idx, double *out_val) {
    if (!v || !out_idx || !out_val || d < 1 || k < 1 || k > d) return -1;
    double *mag = (double *)malloc((size_t)d * sizeof(double));
    int64_t *ord = (int64_t *)malloc((size_t)d * sizeof(int64_t));
    int64_t *tmp = (int64_t *)malloc((size_t)d * sizeof(int64_t));
    if (!mag || !ord || !tmp) { free(mag); free(ord); free(tmp); return -1; }
    for (int64_t j = 0; j < d; ++j) { mag[j] = fabs(v[j]); ord[j] = j; }
    /* bottom-up stable merge sort by magnitude, descending */
    for (int64_t w = 1; w < d; w *= 2) {
        for (int64_t lo = 0; lo < d; lo += 2 * w) {
            int64_t mid = lo + w < d ? lo + w : d;
            int64_t hi = lo + 2 * w < d ? lo + 2 * w : d;
            merge_runs(mag, ord, tmp, lo, mid, hi);
        }
        int64_t *s = ord; ord = tmp; tmp = s;
    }
    qsort(ord, (size_t)k, sizeof(int64_t), cmp_i64); /* the kept positions, ascending */
    for (int64_t r = 0; r < k; ++r) { out_idx[r] = (int32_t)ord[r]; out_val[r] = v[ord[r]]; }
    free(mag); free(ord); free(tmp);
    return 0;
}

/* ------------------------------------------------------------------------------------
 * Objective of Section 5, eq. (9), for ONE worker i holding m data points:
 *   f_i(x) = (1/m) sum_l log(1 + exp(-y_l a_l^T x)) + lambda sum_j x_j^2 / (1 + x_j^2).
 * Reading: eq. (9) is written for the whole data set; each worker's f_i carries the mean
 * loss of its own rows plus the full regulariser, so that (1/n) sum_i f_i is eq. (9) when
 * all workers hold the same number of rows.
 * Gradient (derivative of the above):
 *   grad_j = (1/m) sum_l  -y_l / (1 + exp(y_l a_l^T x)) * a_lj  +  2 lambda x_j / (1 + x_j^2)^2.
 * ------------------------------------------------------------------------------------ */
static double log1pexp_neg(double t) { /* log(1 + exp(-t)) without overflow */
    return t >= 0.0 ? log1p(exp(-t)) : -t + log1p(exp(t));
}

static double regulariser(const double *x, int64_t d, double lambda) {
    double s = 0.0;
    for (int64_t j = 0; j < d; ++j) s += x[j] * x[j] / (1.0 + x[j] * x[j]);
    return lambda * s;
}

static void add_regulariser_grad(const double *x, int64_t d, double lambda, double *grad) {
    for (int64_t j = 0; j < d; ++j) {
        double q = 1.0 + x[j] * x[j];
        grad[j] += 2.0 * lambda * x[j] / (q * q);
    }
}

/* dense rows: A is [m][d] row-major fp32, y is [m] fp32 (+1 / -1) */
double ef21o_logreg_loss_dense(const float *A, const float *y, int64_t m, int64_t d, const double *x,
                               double lambda) {
    double loss = 0.0;
    for (int64_t l = 0; l < m; ++l) {
        double z = 0.0;
        for (int64_t j = 0; j < d; ++j) z += (double)A[l * d + j] * x[j];
        loss += log1pexp_neg((double)y[l] * z);
    }
    return loss / (double)m + regulariser(x, d, lambda);
}

void ef21o_logreg_grad_dense(const float *A, const float *y, int64_t m, int64_t d, const double *x,
                             double lambda, double *grad) {
    for (int64_t j = 0; j < d; ++j) grad[j] = 0.0;
    for (int64_t l = 0; l < m; ++l) {
        double z = 0.0;
        for (int64_t j = 0; j < d; ++j) z += (double)A[l * d + j] * x[j];
        double yl = (double)y[l];
        double r = -yl / (1.0 + exp(yl * z));
        for (int64_t j = 0; j < d; ++j) grad[j] += r * (double)A[l * d + j];
    }
    for (int64_t j = 0; j < d; ++j) grad[j] /= (double)m;
    add_regulariser_grad(x, d, lambda, grad);
}

/* CSR rows: rowptr has m+1 absolute offsets into col/val (rowptr[0] need not be 0) */
double ef21o_logreg_loss_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                             int64_t m, int64_t d, const double *x, double lambda) {
    double loss = 0.0;
    for (int64_t l = 0; l < m; ++l) {
        double z = 0.0;
        for (int64_t p = rowptr[l]; p < rowptr[l + 1]; ++p) z += (double)val[p] * x[col[p]];
        loss += log1pexp_neg((double)y[l] * z);
    }
    return loss / (double)m + regulariser(x, d, lambda);
}

void ef21o_logreg_grad_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                           int64_t m, int64_t d, const double *x, double lambda, double *grad) {
    for (int64_t j = 0; j < d; ++j) grad[j] = 0.0;
    for (int64_t l = 0; l < m; ++l) {
        double z = 0.0;
        for (int64_t p = rowptr[l]; p < rowptr[l + 1]; ++p) z += (double)val[p] * x[col[p]];
        double yl = (double)y[l];
        double r = -yl / (1.0 + exp(yl * z));
        for (int64_t p = rowptr[l]; p < rowptr[l + 1]; ++p) grad[col[p]] += r * (double)val[p];
    }
    for (int64_t j = 0; j < d; ++j) grad[j] /= (double)m;
    add_regulariser_grad(x, d, lambda, grad);
}

/* round a vector to the storage precision in place */
void ef21o_round_storage(double *a, int64_t len, int storage_f32) {
    for (int64_t j = 0; j < len; ++j) a[j] = store(a[j], storage_f32);
}

/* ------------------------------------------------------------------------------------
 * Algorithm 2 (EF21, multiple nodes), the worker loop and the master's aggregation:
 *   line 5:  c_i = C(grad f_i(x) - g_i)          (C = Top-k)
 *   line 6:  g_i <- g_i + c_i
 *   line 8:  g   <- g + (1/n) sum_i c_i
 * grads, g_i: [n][d]; g: [d]; msg_idx, msg_val: [n][k] receive the messages c_i as
 * (ascending index, value) pairs.  The sum over workers in line 8 runs in worker order.
 * Returns 0 on success.
 * ------------------------------------------------------------------------------------ */
int ef21o_compress_update(int32_t n, int64_t d, int64_t k, const double *grads, double *g_i, double *g,
                          int32_t *msg_idx, double *msg_val, int storage_f32) {
    if (n < 1 || d < 1 || k < 1 || k > d) return -1;
    double *v = (double *)malloc((size_t)d * sizeof(double));
    double *sum_c = (double *)calloc((size_t)d, sizeof(double));
    if (!v || !sum_c) { free(v); free(sum_c); return -1; }
    for (int32_t i = 0; i < n; ++i) {
        const double *gr = grads + (int64_t)i * d;
        double *gi = g_i + (int64_t)i * d;
        int32_t *idx = msg_idx + (int64_t)i * k;
        double *val = msg_val + (int64_t)i * k;
        for (int64_t j = 0; j < d; ++j) {
            if (storage_f32) v[j] = (double)((float)gr[j] - (float)gi[j]);
            else v[j] = gr[j] - gi[j];
        }
        if (ef21o_topk(v, d, k, idx, val) != 0) { free(v); free(sum_c); return -1; } /* line 5 */
        for (int64_t r = 0; r < k; ++r) {
            gi[idx[r]] = store(gi[idx[r]] + val[r], storage_f32);                   /* line 6 */
            sum_c[idx[r]] += val[r];
        }
    }
    for (int64_t j = 0; j < d; ++j) g[j] = store(g[j] + sum_c[j] / (double)n, storage_f32); /* line 8 */
    free(v); free(sum_c);
    return 0;
}

/* Algorithm 2, line 3: x <- x - gamma g */
void ef21o_model_step(int64_t d, double gamma, double *x, const double *g, int storage_f32) {
    for (int64_t j = 0; j < d; ++j) x[j] = store(x[j] - gamma * g[j], storage_f32);
}

/* g = (1/n) sum_i g_i  (the input line of Algorithm 2; also the invariant of Section 3.3) */
void ef21o_mean_rows(int32_t n, int64_t d, const double *g_i, double *g, int storage_f32) {
    for (int64_t j = 0; j < d; ++j) {
        double s = 0.0;
        for (int32_t i = 0; i < n; ++i) s += g_i[(int64_t)i * d + j];
        g[j] = store(s / (double)n, storage_f32);
    }
}
