// Local gradients of the objective of Section 5, eq. (9), for all workers:
//   grad f_i(x) = (1/m) sum_l  -y_l / (1 + exp(y_l a_l^T x)) a_l  +  2 lambda x_j / (1 + x_j^2)^2.
//
// These are GEMV-shaped (each matrix entry is used twice, about one flop per byte), far below
// the matrix-core ridge, so they are written as coalesced streaming kernels, not MFMA tiles.
//
// Dense rows, d <= 4096: ONE pass over A.  A wavefront owns whole rows; a lane keeps its columns
// of the row in registers between the dot product (wavefront reduction, no LDS) and the rank-one
// accumulation r_l * a_l into per-lane accumulators.  Workgroups write partial sums that a small
// second kernel adds in a fixed order (bitwise reproducible), together with the regulariser.
// Dense rows, larger d: z = A x, then A^T r, two passes.  (CSR rows: logreg_csr.hip.)
#include "device_utils.h"
#include "kernels.h"
#include "logreg_finish.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

struct DensePlan {
    int64_t rows_per_wg;
    int64_t chunks;   // workgroups (row blocks) per worker
};

// About two workgroups per compute unit in all (512 on 256 CUs), each streaming one long block of rows:
// fewer, longer blocks measured faster than several rounds of short ones, and they leave fewer partial
// sums to add.  At least 8 rows each.
DensePlan dense_plan(int32_t n, int64_t m) {
    int64_t target = 512 / n;
    if (target < 1) target = 1;
    int64_t rows = (m + target - 1) / target;
    if (rows < 8) rows = 8;
    return {rows, (m + rows - 1) / rows};
}

// No batch of tau <= m rows gets more workgroups per worker than this (the partial sums are sized by it).
int64_t max_chunks(int32_t n, int64_t m) {
    int64_t target = 512 / n;
    if (target < 1) target = 1;
    const int64_t by_rows = (m + 7) / 8;
    return by_rows < target ? by_rows : target;
}

// Row `l` of a worker's batch: the row of A it names, or -1 when the entry lies outside [0, m_full) (such an
// entry contributes nothing and is never dereferenced).
__device__ __forceinline__ int64_t batch_row(const int32_t *__restrict__ batch, int64_t at, int64_t m_full) {
    const uint32_t b = (uint32_t)batch[at];
    return b < (uint64_t)m_full ? (int64_t)b : -1;
}

// ------------------------------------------------------------------ dense, one pass over A
// BATCH: the m rows of a worker are the entries of batch[worker][0..m) (row numbers inside its m_full rows), the
// minibatch of Algorithm 5; otherwise m_full == m and row l is row l.
template <int VEC, int NQ, int ROWS, bool BATCH>
__global__ __launch_bounds__(kThreads) void logreg_dense_fused_kernel(const float *__restrict__ A,
                                                                      const float *__restrict__ y,
                                                                      const float *__restrict__ x,
                                                                      float *__restrict__ part, int64_t m,
                                                                      int64_t d, int64_t rows_per_wg, int loss,
                                                                      const int32_t *__restrict__ batch,
                                                                      int64_t m_full, int64_t x_stride) {
    constexpr int kCols = NQ * kWave * VEC;   // columns covered by one wavefront
    __shared__ float red[kCols];
    const int64_t worker = blockIdx.y, chunk = blockIdx.x, chunks = gridDim.x;
    x += worker * x_stride;                   // 0: one x for all workers
    const int wave = threadIdx.x / kWave, lane = lane_id();

    float xr[NQ][VEC], acc[NQ][VEC];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int64_t c0 = ((int64_t)q * kWave + lane) * VEC;
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            xr[q][t] = (c0 + t < d) ? x[c0 + t] : 0.f;
            acc[q][t] = 0.f;
        }
    }

    // ROWS rows per wavefront and trip: their loads are all issued before the first dot product.  A row
    // index past the block is clamped to the block's last row and its coefficient set to zero.
    const int64_t l0 = chunk * rows_per_wg;
    const int64_t l1 = l0 + rows_per_wg < m ? l0 + rows_per_wg : m;
    for (int64_t l = l0 + wave * ROWS; l < l1; l += kWaves * ROWS) {
        float av[ROWS][NQ][VEC], yl[ROWS], s[ROWS];
        bool live[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            int64_t lr = l + r < l1 ? l + r : l1 - 1;
            live[r] = l + r < l1;
            if constexpr (BATCH) {
                lr = batch_row(batch, worker * m + lr, m_full);
                if (lr < 0) {
                    lr = 0;
                    live[r] = false;
                }
            }
            const float *row = A + (worker * m_full + lr) * d;
            yl[r] = y[worker * m_full + lr];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int64_t c0 = ((int64_t)q * kWave + lane) * VEC;
                if constexpr (VEC == 4) {
                    float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (c0 < d) t4 = stream_load4(row + c0);
                    av[r][q][0] = t4.x;
                    av[r][q][1] = t4.y;
                    av[r][q][2] = t4.z;
                    av[r][q][3] = t4.w;
                } else {
                    av[r][q][0] = (c0 < d) ? stream_load(row + c0) : 0.f;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            s[r] = 0.f;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < VEC; ++t) s[r] = fmaf(av[r][q][t], xr[q][t], s[r]);
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) s[r] = wave_sum(s[r]);
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const float coef = live[r] ? loss_derivative(yl[r], s[r], loss) : 0.f;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < VEC; ++t) acc[q][t] = fmaf(coef, av[r][q][t], acc[q][t]);
        }
    }

    // add the four wavefronts' accumulators in wavefront order
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int t = 0; t < VEC; ++t) {
                    const int c = (q * kWave + lane) * VEC + t;
                    red[c] = (w == 0 ? 0.f : red[c]) + acc[q][t];
                }
        }
        __syncthreads();
    }
    float *out = part + (worker * chunks + chunk) * d;
    for (int c = threadIdx.x; c < kCols && c < d; c += kThreads) out[c] = red[c];
}

// ------------------------------------------------------------------ dense, any d: two passes
__global__ __launch_bounds__(kThreads) void logreg_dense_residual_kernel(const float *__restrict__ A,
                                                                         const float *__restrict__ y,
                                                                         const float *__restrict__ x,
                                                                         float *__restrict__ r, int64_t rows,
                                                                         int64_t d, int loss, int64_t m,
                                                                         const int32_t *__restrict__ batch,
                                                                         int64_t m_full, int64_t x_stride) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t l = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; l < rows; l += nwaves) {
        int64_t src = l;                        // rows counts n * m entries; with a batch, m of m_full rows each
        if (batch) {
            const int64_t b = batch_row(batch, l, m_full);
            if (b < 0) {
                if (lane == 0) r[l] = 0.f;
                continue;
            }
            src = (l / m) * m_full + b;
        }
        const float *row = A + src * d;
        const float *xw = x + (l / m) * x_stride;
        float s = 0.f;
        for (int64_t c = lane; c < d; c += kWave) s = fmaf(row[c], xw[c], s);
        s = wave_sum(s);
        if (lane == 0) r[l] = loss_derivative(y[src], s, loss);
    }
}

__global__ __launch_bounds__(kThreads) void logreg_dense_atr_kernel(const float *__restrict__ A,
                                                                    const float *__restrict__ r,
                                                                    float *__restrict__ part, int64_t m, int64_t d,
                                                                    int64_t rows_per_wg,
                                                                    const int32_t *__restrict__ batch,
                                                                    int64_t m_full) {
    const int64_t worker = blockIdx.z, chunk = blockIdx.y, chunks = gridDim.y;
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c >= d) return;
    const int64_t l0 = chunk * rows_per_wg;
    const int64_t l1 = l0 + rows_per_wg < m ? l0 + rows_per_wg : m;
    float acc = 0.f;
    for (int64_t l = l0; l < l1; ++l) {
        int64_t src = l;
        if (batch) {
            src = batch_row(batch, worker * m + l, m_full);
            if (src < 0) continue;              // its residual is zero as well
        }
        acc = fmaf(r[worker * m + l], A[(worker * m_full + src) * d + c], acc);
    }
    part[(worker * chunks + chunk) * d + c] = acc;
}

// grad[i][j] from the partial sums: one thread per (worker, column).
__global__ __launch_bounds__(kThreads) void logreg_dense_finish_kernel(const float *__restrict__ part,
                                                                       const float *__restrict__ x,
                                                                       float *__restrict__ grad, int64_t chunks,
                                                                       int64_t m, int64_t d, float lambda,
                                                                       int64_t x_stride) {
    const int64_t worker = blockIdx.y;
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c < d)
        grad[worker * d + c] =
            dense_grad_entry(part + worker * chunks * d, chunks, d, c, x[worker * x_stride + c], m, lambda);
}

struct DenseArgs {
    const float *A, *y, *x;
    float *part;
    int32_t n;
    int64_t m, d;          // m: rows summed per worker (the batch size under a batch)
    DensePlan pl;
    int loss;
    const int32_t *batch;
    int64_t m_full, x_stride;
};

template <int VEC, int NQ>
void launch_fused(const DenseArgs &a, hipStream_t stream) {
    constexpr int ROWS = NQ * VEC <= 32 ? 2 : 1;     // two rows in flight while their registers fit
    const dim3 grid((unsigned)a.pl.chunks, (unsigned)a.n);
    if (a.batch)
        hipLaunchKernelGGL((logreg_dense_fused_kernel<VEC, NQ, ROWS, true>), grid, dim3(kThreads), 0, stream, a.A, a.y,
                           a.x, a.part, a.m, a.d, a.pl.rows_per_wg, a.loss, a.batch, a.m_full, a.x_stride);
    else
        hipLaunchKernelGGL((logreg_dense_fused_kernel<VEC, NQ, ROWS, false>), grid, dim3(kThreads), 0, stream, a.A, a.y,
                           a.x, a.part, a.m, a.d, a.pl.rows_per_wg, a.loss, a.batch, a.m_full, a.x_stride);
}

}  // namespace

size_t logreg_dense_scratch_bytes(int32_t n, int64_t m, int64_t d) {
    return sizeof(float) * ((size_t)n * max_chunks(n, m) * d + (size_t)n * m);   // partial sums + residuals
}

hipError_t launch_logreg_grad_dense(const float *A, const float *y, const float *x, float *grad, int32_t n,
                                    int64_t m_full, int64_t d, float lambda, void *scratch, hipStream_t stream,
                                    const Marker &mk, GradParts *defer, int loss, RowBatch rb, int64_t x_stride) {
    if (defer) *defer = GradParts();
    const int32_t *batch = rb.tau > 0 ? rb.rows : nullptr;
    const int64_t m = batch ? rb.tau : m_full;         // rows summed per worker (tau <= m_full, checked by the caller)
    const DensePlan pl = dense_plan(n, m);
    float *part = (float *)scratch;
    float *resid = part + (size_t)n * max_chunks(n, m_full) * d;
    const bool vec4 = (d % 4 == 0) && ((uintptr_t)A % 16 == 0);
    const DenseArgs a{A, y, x, part, n, m, d, pl, loss, batch, m_full, x_stride};
    bool fused = true;
    if (vec4 && d <= 256) launch_fused<4, 1>(a, stream);
    else if (vec4 && d <= 512) launch_fused<4, 2>(a, stream);
    else if (vec4 && d <= 1024) launch_fused<4, 4>(a, stream);
    else if (vec4 && d <= 2048) launch_fused<4, 8>(a, stream);
    else if (vec4 && d <= 4096) launch_fused<4, 16>(a, stream);
    else if (d <= 128) launch_fused<1, 2>(a, stream);
    else if (d <= 512) launch_fused<1, 8>(a, stream);
    else if (d <= 2048) launch_fused<1, 32>(a, stream);
    else fused = false;
    if (!fused) {
        const int64_t rows = (int64_t)n * m;
        int64_t blocks = (rows + kWaves - 1) / kWaves;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(logreg_dense_residual_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, A, y, x,
                           resid, rows, d, loss, m, batch, m_full, x_stride);
        hipLaunchKernelGGL(logreg_dense_atr_kernel,
                           dim3((unsigned)((d + kThreads - 1) / kThreads), (unsigned)pl.chunks, (unsigned)n),
                           dim3(kThreads), 0, stream, A, resid, part, m, d, pl.rows_per_wg, batch, m_full);
    }
    mk(K_GRAD_MAIN);
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return st;
    if (defer && fused && x_stride == 0) {      // the consumer finishes the sums itself (dense_grad_entry)
        *defer = GradParts{part, pl.chunks, m, x, lambda};
        return hipSuccess;
    }
    hipLaunchKernelGGL(logreg_dense_finish_kernel, dim3((unsigned)((d + kThreads - 1) / kThreads), (unsigned)n),
                       dim3(kThreads), 0, stream, part, x, grad, pl.chunks, m, d, lambda, x_stride);
    mk(K_GRAD_AUX);
    return hipGetLastError();
}

}  // namespace ef21
