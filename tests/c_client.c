/*
 * A client of libef21.so written in plain C (C99): it includes include/ef21.h, links the library and the HIP
 * runtime, and checks, against a brute-force selection of its own on the host,
 *   1. ef21_topk and ef21_topk_static on three long rows (Section 2.1: the k entries of largest magnitude, lower
 *      index first among equal magnitudes, positions ascending), bit for bit;
 *   2. one iteration of Algorithm 2 from the zero state with supplied gradients: the messages are the Top-k of
 *      the gradients (line 5 with g_i = 0), g_i holds exactly those entries (line 6), g = (1/n) sum_i c_i
 *      (line 8) and x = -gamma g (line 3), the last two within fp32 rounding.
 * Prints one line per check and returns 0 if all hold.  Built by paper_2106_05203_amd/build.py, run by
 * tests/test_gpu_c_client.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ef21.h"

#define HIP_OK(call)                                                                              \
    do {                                                                                          \
        hipError_t st_ = (call);                                                                  \
        if (st_ != hipSuccess) {                                                                  \
            fprintf(stderr, "%s:%d: %s: %s\n", __FILE__, __LINE__, #call, hipGetErrorString(st_)); \
            return 2;                                                                             \
        }                                                                                         \
    } while (0)

#define EF21_CALL(call)                                                                  \
    do {                                                                                 \
        int rc_ = (call);                                                                \
        if (rc_ != EF21_OK) {                                                            \
            fprintf(stderr, "%s:%d: %s: %d %s\n", __FILE__, __LINE__, #call, rc_, ef21_last_error()); \
            return 2;                                                                    \
        }                                                                                \
    } while (0)

enum { N = 3, K = 500 };
static const int64_t D = 70001;

static uint32_t mix(uint32_t v) {
    v ^= v >> 16;
    v *= 0x7feb352dU;
    v ^= v >> 15;
    v *= 0x846ca68bU;
    v ^= v >> 16;
    return v;
}

static const float *sort_row;
static int by_magnitude_then_position(const void *pa, const void *pb) {
    const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    const float ma = fabsf(sort_row[a]), mb = fabsf(sort_row[b]);
    if (ma != mb) return ma > mb ? -1 : 1;
    return a < b ? -1 : (a > b ? 1 : 0);
}
static int ascending(const void *pa, const void *pb) {
    const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

/* the k entries of largest magnitude of row (lower index first among equals), positions ascending */
static void host_topk(const float *row, int64_t d, int k, int32_t *idx, float *val, int32_t *order) {
    for (int64_t j = 0; j < d; ++j) order[j] = (int32_t)j;
    sort_row = row;
    qsort(order, (size_t)d, sizeof(int32_t), by_magnitude_then_position);
    memcpy(idx, order, sizeof(int32_t) * (size_t)k);
    qsort(idx, (size_t)k, sizeof(int32_t), ascending);
    for (int t = 0; t < k; ++t) val[t] = row[idx[t]];
}

int main(void) {
    const size_t row_bytes = sizeof(float) * (size_t)D;
    float *rows = (float *)malloc(row_bytes * N);
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)D);
    int32_t *ref_idx = (int32_t *)malloc(sizeof(int32_t) * N * K), *got_idx = (int32_t *)malloc(sizeof(int32_t) * N * K);
    float *ref_val = (float *)malloc(sizeof(float) * N * K), *got_val = (float *)malloc(sizeof(float) * N * K);
    float *g_i = (float *)malloc(row_bytes * N), *g = (float *)malloc(row_bytes), *x = (float *)malloc(row_bytes);
    if (!rows || !order || !ref_idx || !got_idx || !ref_val || !got_val || !g_i || !g || !x) return 2;
    /* magnitudes on a grid of 20 011 values (so some are equal), random signs */
    for (int i = 0; i < N; ++i)
        for (int64_t j = 0; j < D; ++j) {
            const uint32_t h = mix((uint32_t)(i * D + j) + 12345u);
            const float mag = (float)(1u + h % 20011u) * 0.001f;
            rows[i * D + j] = (h >> 31) ? -mag : mag;
        }
    for (int i = 0; i < N; ++i) host_topk(rows + i * D, D, K, ref_idx + i * K, ref_val + i * K, order);

    float *d_rows = NULL, *d_val = NULL;
    int32_t *d_idx = NULL;
    HIP_OK(hipMalloc((void **)&d_rows, row_bytes * N));
    HIP_OK(hipMalloc((void **)&d_idx, sizeof(int32_t) * N * K));
    HIP_OK(hipMalloc((void **)&d_val, sizeof(float) * N * K));
    HIP_OK(hipMemcpy(d_rows, rows, row_bytes * N, hipMemcpyHostToDevice));

    int failures = 0;
    for (int variant = 0; variant < 2; ++variant) {
        HIP_OK(hipMemset(d_idx, 0xff, sizeof(int32_t) * N * K));
        HIP_OK(hipMemset(d_val, 0xff, sizeof(float) * N * K));
        if (variant == 0) EF21_CALL(ef21_topk(d_rows, N, D, K, d_idx, d_val, NULL));
        else EF21_CALL(ef21_topk_static(d_rows, N, D, K, d_idx, d_val, NULL));
        HIP_OK(hipDeviceSynchronize());
        HIP_OK(hipMemcpy(got_idx, d_idx, sizeof(int32_t) * N * K, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(got_val, d_val, sizeof(float) * N * K, hipMemcpyDeviceToHost));
        const int same = memcmp(got_idx, ref_idx, sizeof(int32_t) * N * K) == 0 &&
                         memcmp(got_val, ref_val, sizeof(float) * N * K) == 0;
        printf("%s: %s\n", variant == 0 ? "ef21_topk" : "ef21_topk_static", same ? "ok" : "MISMATCH");
        failures += !same;
    }

    const float gamma = 0.5f;
    ef21_handle h = ef21_create(N, D, K, gamma);
    if (!h) {
        fprintf(stderr, "ef21_create: %s\n", ef21_last_error());
        return 2;
    }
    EF21_CALL(ef21_step(h, d_rows, EF21_ORDER_GRAD_FIRST));
    HIP_OK(hipDeviceSynchronize());
    EF21_CALL(ef21_get_messages(h, d_idx, d_val));
    float *d_x = NULL, *d_gi = NULL, *d_g = NULL;
    HIP_OK(hipMalloc((void **)&d_x, row_bytes));
    HIP_OK(hipMalloc((void **)&d_gi, row_bytes * N));
    HIP_OK(hipMalloc((void **)&d_g, row_bytes));
    EF21_CALL(ef21_get_state(h, d_x, d_gi, d_g));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(got_idx, d_idx, sizeof(int32_t) * N * K, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(got_val, d_val, sizeof(float) * N * K, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(x, d_x, row_bytes, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(g_i, d_gi, row_bytes * N, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(g, d_g, row_bytes, hipMemcpyDeviceToHost));
    {
        const int same = memcmp(got_idx, ref_idx, sizeof(int32_t) * N * K) == 0 &&
                         memcmp(got_val, ref_val, sizeof(float) * N * K) == 0;
        printf("messages of the first iteration: %s\n", same ? "ok" : "MISMATCH");
        failures += !same;
    }
    {
        /* line 6: g_i = C(grad f_i) exactly; lines 8 and 3 within fp32 rounding of sums of at most N terms */
        double *sum = (double *)calloc((size_t)D, sizeof(double)), *sum_abs = (double *)calloc((size_t)D, sizeof(double));
        float *dense = (float *)calloc((size_t)D, sizeof(float));
        if (!sum || !sum_abs || !dense) return 2;
        int gi_ok = 1, g_ok = 1, x_ok = 1;
        for (int i = 0; i < N; ++i) {
            memset(dense, 0, row_bytes);
            for (int t = 0; t < K; ++t) {
                const int32_t j = ref_idx[i * K + t];
                dense[j] = ref_val[i * K + t];
                sum[j] += (double)ref_val[i * K + t];
                sum_abs[j] += fabs((double)ref_val[i * K + t]);
            }
            gi_ok = gi_ok && memcmp(dense, g_i + i * D, row_bytes) == 0;
        }
        const double u = 1.0 / 16777216.0; /* 2^-24 */
        for (int64_t j = 0; j < D; ++j) {
            const double g_ref = sum[j] / N, x_ref = -(double)gamma * g_ref;
            const double tol_g = 1e-5 * fabs(g_ref) + (N + 2) * u * sum_abs[j] / N;
            g_ok = g_ok && fabs((double)g[j] - g_ref) <= tol_g;
            x_ok = x_ok && fabs((double)x[j] - x_ref) <= 1e-5 * fabs(x_ref) + gamma * tol_g + 2 * u * fabs(x_ref);
        }
        printf("g_i after line 6: %s\ng after line 8: %s\nx after line 3: %s\n", gi_ok ? "ok" : "MISMATCH",
               g_ok ? "ok" : "MISMATCH", x_ok ? "ok" : "MISMATCH");
        failures += !gi_ok + !g_ok + !x_ok;
        free(sum);
        free(sum_abs);
        free(dense);
    }
    EF21_CALL(ef21_destroy(h));
    HIP_OK(hipFree(d_rows));
    HIP_OK(hipFree(d_idx));
    HIP_OK(hipFree(d_val));
    HIP_OK(hipFree(d_x));
    HIP_OK(hipFree(d_gi));
    HIP_OK(hipFree(d_g));
    free(rows); free(order); free(ref_idx); free(got_idx); free(ref_val); free(got_val); free(g_i); free(g); free(x);
    if (failures) printf("c_client: %d checks failed\n", failures);
    else printf("c_client: all checks passed\n");
    return failures ? 1 : 0;
}
