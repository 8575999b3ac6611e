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
#include "logreg_dense_block.h"
#include "logreg_finish.h"

namespace ef21 {
namespace {

constexpr int kThreads = kDenseThreads;
constexpr int kWaves = kDenseWaves;

// ------------------------------------------------------------------ dense, one pass over A
template <int VEC, int NQ, int ROWS, bool BATCH>
__global__ __launch_bounds__(kThreads) void logreg_dense_fused_kernel(const float *__restrict__ A,
                                                                      const float *__restrict__ y,
                                                                      const float *__restrict__ x,
                                                                      float *__restrict__ part, int64_t m,
                                                                      int64_t d, int64_t rows_per_wg, int loss,
                                                                      const int32_t *__restrict__ batch,
                                                                      int64_t m_full, int64_t x_stride) {
    __shared__ float red[NQ * kWave * VEC];
    const int64_t worker = blockIdx.y;
    dense_block<VEC, NQ, ROWS, BATCH>(A, y, x + worker * x_stride /* 0: one x for all workers */, part, m, d,
                                      rows_per_wg, loss, batch, m_full, worker, blockIdx.x, gridDim.x,
                                      threadIdx.x / kWave, threadIdx.x, true, red);
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
    constexpr int ROWS = dense_rows_in_flight<VEC, NQ>();
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
    const DenseVariant dv = dense_variant(d, vec4);
    const bool fused = dv.vec != 0;
    switch (dv.vec * 100 + dv.nq) {
        case 401: launch_fused<4, 1>(a, stream); break;
        case 402: launch_fused<4, 2>(a, stream); break;
        case 404: launch_fused<4, 4>(a, stream); break;
        case 408: launch_fused<4, 8>(a, stream); break;
        case 416: launch_fused<4, 16>(a, stream); break;
        case 102: launch_fused<1, 2>(a, stream); break;
        case 108: launch_fused<1, 8>(a, stream); break;
        case 132: launch_fused<1, 32>(a, stream); break;
        default: break;
    }
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
