// Local gradients of the objective of Section 5, eq. (9), for all workers, sparse (CSR) rows:
//   grad f_i(x) = (1/m) sum_l  -y_l / (1 + exp(y_l a_l^T x)) a_l  +  2 lambda x_j / (1 + x_j^2)^2.
//
// Both halves of this computation are 4-byte random accesses into a d-vector per worker (gather from
// x, scatter-add into the gradient).  Served from L2 they move a whole cache line per entry and are
// an order of magnitude off the bandwidth roofline (and global float atomics are worse still), so
// the vector is held in LDS instead.  A few workgroups must share a CU, hence the columns are cut into
// R = ceil(d / 12288) ranges, and when the column indices of every row are ascending (checked once,
// when the problem is attached) a range's slice of each row is contiguous and found through an index
// built at attach time.  Two streaming passes over the non-zeros, one workgroup per (range, worker):
//   pass 1  x-range in LDS; one wavefront per row slice: partial dot product z_part[range][row]
//   pass 2  coef_l = r_l / m from the summed partial dot products; r_l * a_l accumulated with LDS
//           atomics in a range-sized LDS buffer, written out once together with the regulariser term
// Unsorted rows, or d too large for the index, fall back to a kernel built on global atomics.
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kAtrThreads = 1024;
constexpr int kAtrWaves = kAtrThreads / kWave;
constexpr int kRangeCols = 12288;     // at most this many columns per range (48 KB of LDS as fp32)
constexpr int kMaxRanges = 64;

__device__ __forceinline__ float residual(float y, float z) {   // -y / (1 + exp(y z))
    return -y / (1.0f + expf(y * z));
}

__device__ __forceinline__ float regulariser_grad(float xj, float lambda) {
    const float q = 1.0f + xj * xj;
    return 2.0f * lambda * xj / (q * q);
}

struct IndexLayout {
    uint32_t *bad;      // [64] count of rows that are not ascending / out of range (first word)
    float *zpart;       // [R][rows] partial dot products of pass 1
    int32_t *split;     // [R + 1][rows] offsets of the column ranges inside each row
    int R;
    int64_t Wc;
};

size_t index_layout(int32_t n, int64_t m, int64_t d, char *base, IndexLayout *out) {
    int64_t R = (d + kRangeCols - 1) / kRangeCols;
    if (R < 1) R = 1;
    int64_t Wc = ((d + R - 1) / R + 63) / 64 * 64;
    const int64_t rows = (int64_t)n * m;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    char *b = take(256);
    char *c = take(sizeof(float) * (size_t)rows * R);
    char *s = take(sizeof(int32_t) * (size_t)rows * (R + 1));   // [R + 1][rows]
    if (out) {
        out->bad = (uint32_t *)b;
        out->zpart = (float *)c;
        out->split = (int32_t *)s;
        out->R = (int)R;
        out->Wc = Wc;
    }
    return off;
}

bool index_possible(int64_t d) { return (d + kRangeCols - 1) / kRangeCols <= kMaxRanges; }

// ---- attach time
__global__ __launch_bounds__(kThreads) void csr_inspect_kernel(const int64_t *__restrict__ rowptr,
                                                               const int32_t *__restrict__ col, int64_t rows,
                                                               int64_t d, uint32_t *bad) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t l = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; l < rows; l += nwaves) {
        const int64_t p0 = rowptr[l], p1 = rowptr[l + 1];
        bool wrong = p1 < p0 || p1 - p0 > 0x7fffffff;
        for (int64_t p = p0 + lane; p < p1; p += kWave) {
            const int32_t c = col[p];
            if (c < 0 || c >= d) wrong = true;
            if (p > p0 && col[p - 1] >= c) wrong = true;
        }
        if (__ballot(wrong) != 0 && lane == 0) atomicAdd(bad, 1u);
    }
}

__global__ __launch_bounds__(kThreads) void csr_split_kernel(const int64_t *__restrict__ rowptr,
                                                             const int32_t *__restrict__ col, int64_t rows, int R,
                                                             int64_t Wc, int32_t *__restrict__ split) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t l = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; l < rows; l += nwaves) {
        const int64_t p0 = rowptr[l], p1 = rowptr[l + 1];
        for (int c = 1; c < R; ++c) {       // entries below the start of range c
            uint32_t below = 0;
            for (int64_t p = p0 + lane; p < p1; p += kWave) below += col[p] < c * Wc ? 1u : 0u;
#pragma unroll
            for (int o = kWave / 2; o > 0; o >>= 1) below += __shfl_xor(below, o, kWave);
            if (lane == 0) split[(int64_t)c * rows + l] = (int32_t)below;
        }
        if (lane == 0) {
            split[l] = 0;
            split[(int64_t)R * rows + l] = (int32_t)(p1 - p0);
        }
    }
}

// Both passes walk a worker's rows kRows at a time per wavefront: lanes 0..kRows-1 fetch the bounds
// of the rows' slices (split is [R + 1][rows]), the bounds are broadcast, and the slices' loads are
// issued for all kRows rows before anything is consumed -- a row slice is short (d/R times the
// density, typically one or two loads per lane), so one row at a time would leave a wavefront
// waiting on a chain of dependent loads per row.  Addresses past a slice's end are clamped to its
// last entry and their contribution dropped, so that no load sits behind a branch.
constexpr int kRows = 8;

struct SliceBounds {
    int64_t b;      // first entry of the slice (lane u holds row u of the batch)
    int32_t len;
};

__device__ __forceinline__ SliceBounds batch_bounds(const int64_t *rowptr, const int32_t *split, int64_t rows,
                                                    int range, int64_t worker, int64_t m, int64_t l0, int lane) {
    const int u = lane & (kRows - 1);
    const bool valid = l0 + u < m;
    const int64_t row = worker * m + (valid ? l0 + u : m - 1);
    const int32_t s0 = split[(int64_t)range * rows + row];
    SliceBounds sb;
    sb.b = rowptr[row] + s0;
    sb.len = valid ? split[(int64_t)(range + 1) * rows + row] - s0 : 0;
    return sb;
}

__device__ __forceinline__ int32_t batch_longest(int32_t len) {
#pragma unroll
    for (int o = kRows / 2; o > 0; o >>= 1) {
        const int32_t other = __shfl_xor(len, o, kWave);
        len = other > len ? other : len;
    }
    return __shfl(len, 0, kWave);
}

// ---- pass 1: partial dot products.  Dynamic LDS: Wc floats.
__global__ __launch_bounds__(kAtrThreads) void csr_dot_kernel(const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col,
                                                              const float *__restrict__ val,
                                                              const int32_t *__restrict__ split,
                                                              const float *__restrict__ x, float *__restrict__ zpart,
                                                              int64_t m, int64_t d, int64_t Wc) {
    extern __shared__ float lds[];
    const int range = blockIdx.x;
    const int64_t worker = blockIdx.y, rows = (int64_t)gridDim.y * m;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t c0 = (int64_t)range * Wc;
    const int64_t width = c0 + Wc < d ? Wc : d - c0;
    for (int64_t j = threadIdx.x; j < width; j += kAtrThreads) lds[j] = x[c0 + j];
    __syncthreads();
    for (int64_t l0 = (int64_t)wave * kRows; l0 < m; l0 += (int64_t)kAtrWaves * kRows) {
        const SliceBounds mine = batch_bounds(rowptr, split, rows, range, worker, m, l0, lane);
        const int32_t longest = batch_longest(mine.len);
        float s[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) s[u] = 0.f;
        for (int32_t t0 = 0; t0 < longest; t0 += kWave) {
            int32_t c[kRows];
            float v[kRows];
            bool in[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int64_t b = __shfl(mine.b, u, kWave);
                const int32_t len = __shfl(mine.len, u, kWave);
                in[u] = t0 + lane < len;
                const int64_t at = b + (in[u] ? t0 + lane : (len > 0 ? len - 1 : 0));
                c[u] = len > 0 ? stream_load(col + at) : (int32_t)c0;
                v[u] = len > 0 ? stream_load(val + at) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const float xv = lds[c[u] - c0];
                if (in[u]) s[u] = fmaf(v[u], xv, s[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const float z = wave_sum(s[u]);
            if (lane == 0 && l0 + u < m) zpart[(int64_t)range * rows + worker * m + l0 + u] = z;
        }
    }
}

// ---- pass 2: gradient of one column range.  Dynamic LDS: Wc floats.
__global__ __launch_bounds__(kAtrThreads) void csr_atr_kernel(const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col,
                                                              const float *__restrict__ val,
                                                              const float *__restrict__ y,
                                                              const float *__restrict__ zpart,
                                                              const int32_t *__restrict__ split,
                                                              const float *__restrict__ x, float *__restrict__ grad,
                                                              int64_t m, int64_t d, int R, int64_t Wc, float lambda) {
    extern __shared__ float lds[];
    const int range = blockIdx.x;
    const int64_t worker = blockIdx.y, rows = (int64_t)gridDim.y * m;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t c0 = (int64_t)range * Wc;
    const int64_t width = c0 + Wc < d ? Wc : d - c0;
    for (int64_t j = threadIdx.x; j < width; j += kAtrThreads) lds[j] = 0.f;
    __syncthreads();
    const float inv_m = 1.0f / (float)m;
    for (int64_t l0 = (int64_t)wave * kRows; l0 < m; l0 += (int64_t)kAtrWaves * kRows) {
        const SliceBounds mine = batch_bounds(rowptr, split, rows, range, worker, m, l0, lane);
        const int32_t longest = batch_longest(mine.len);
        // coef_l = r_l / m of "my" row of the batch: the partial dot products are added in range order
        const int64_t my_row = worker * m + (l0 + (lane & (kRows - 1)) < m ? l0 + (lane & (kRows - 1)) : m - 1);
        float z = 0.f;
        for (int r = 0; r < R; ++r) z += zpart[(int64_t)r * rows + my_row];
        const float my_cf = residual(y[my_row], z) * inv_m;
        for (int32_t t0 = 0; t0 < longest; t0 += kWave) {
            int32_t c[kRows];
            float v[kRows];
            bool in[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int64_t b = __shfl(mine.b, u, kWave);
                const int32_t len = __shfl(mine.len, u, kWave);
                in[u] = t0 + lane < len;
                const int64_t at = b + (in[u] ? t0 + lane : (len > 0 ? len - 1 : 0));
                c[u] = len > 0 ? stream_load(col + at) : (int32_t)c0;
                v[u] = len > 0 ? stream_load(val + at) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const float cf = __shfl(my_cf, u, kWave);
                if (in[u]) atomicAdd(&lds[c[u] - c0], cf * v[u]);
            }
        }
    }
    __syncthreads();
    for (int64_t j = threadIdx.x; j < width; j += kAtrThreads)
        grad[worker * d + c0 + j] = lds[j] + regulariser_grad(x[c0 + j], lambda);
}

// ---- fallback: global atomics, any column order
__global__ __launch_bounds__(kThreads) void csr_regulariser_kernel(const float *__restrict__ x,
                                                                   float *__restrict__ grad, int64_t d,
                                                                   float lambda) {
    const int64_t worker = blockIdx.y;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c < d; c += stride)
        grad[worker * d + c] = regulariser_grad(x[c], lambda);
}

__global__ __launch_bounds__(kThreads) void csr_atomic_kernel(const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col,
                                                              const float *__restrict__ val,
                                                              const float *__restrict__ y,
                                                              const float *__restrict__ x, float *grad, int64_t rows,
                                                              int64_t m, int64_t d, float inv_m) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t l = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; l < rows; l += nwaves) {
        const int64_t p0 = rowptr[l], p1 = rowptr[l + 1];
        float s = 0.f;
        // a column index outside [0, d) is skipped rather than dereferenced
        for (int64_t p = p0 + lane; p < p1; p += kWave) {
            const uint32_t c = (uint32_t)col[p];
            if (c < (uint64_t)d) s = fmaf(val[p], x[c], s);
        }
        s = wave_sum(s);
        const float coef = residual(y[l], s) * inv_m;
        float *g = grad + (l / m) * d;
        for (int64_t p = p0 + lane; p < p1; p += kWave) {
            const uint32_t c = (uint32_t)col[p];
            if (c < (uint64_t)d) atomicAdd(g + c, coef * val[p]);
        }
    }
}

unsigned row_blocks(int64_t rows) {
    int64_t blocks = (rows + kWaves - 1) / kWaves;
    if (blocks > 16384) blocks = 16384;
    return (unsigned)blocks;
}

}  // namespace

size_t logreg_csr_index_bytes(int32_t n, int64_t m, int64_t d) {
    return index_possible(d) ? index_layout(n, m, d, nullptr, nullptr) : 0;
}

hipError_t logreg_csr_build_index(const int64_t *rowptr, const int32_t *col, int32_t n, int64_t m, int64_t d,
                                  void *index, hipStream_t stream, bool *usable) {
    *usable = false;
    if (!index || !index_possible(d)) return hipSuccess;
    IndexLayout ix;
    index_layout(n, m, d, (char *)index, &ix);
    const int64_t rows = (int64_t)n * m;
    hipError_t st = hipMemsetAsync(ix.bad, 0, 256, stream);
    if (st != hipSuccess) return st;
    hipLaunchKernelGGL(csr_inspect_kernel, dim3(row_blocks(rows)), dim3(kThreads), 0, stream, rowptr, col, rows, d,
                       ix.bad);
    uint32_t bad = 0;
    st = hipMemcpyAsync(&bad, ix.bad, sizeof(bad), hipMemcpyDeviceToHost, stream);
    if (st != hipSuccess) return st;
    st = hipStreamSynchronize(stream);
    if (st != hipSuccess) return st;
    if (bad != 0) return hipSuccess;      // not ascending everywhere: the caller uses the atomic kernel
    hipLaunchKernelGGL(csr_split_kernel, dim3(row_blocks(rows)), dim3(kThreads), 0, stream, rowptr, col, rows, ix.R,
                       ix.Wc, ix.split);
    st = hipStreamSynchronize(stream);
    if (st != hipSuccess) return st;
    *usable = true;
    return hipGetLastError();
}

hipError_t launch_logreg_grad_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                                  const float *x, float *grad, int32_t n, int64_t m, int64_t d, float lambda,
                                  const void *index, hipStream_t stream, const Marker &mk) {
    const int64_t rows = (int64_t)n * m;
    if (index) {
        IndexLayout ix;
        index_layout(n, m, d, (char *)const_cast<void *>(index), &ix);
        const size_t lds_bytes = sizeof(float) * (size_t)ix.Wc;
        static bool configured = false;
        if (!configured) {
            hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csr_dot_kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kRangeCols);
            if (st == hipSuccess)
                st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csr_atr_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kRangeCols);
            if (st != hipSuccess) return st;
            configured = true;
        }
        const dim3 grid((unsigned)ix.R, (unsigned)n), block(kAtrThreads);
        hipLaunchKernelGGL(csr_dot_kernel, grid, block, lds_bytes, stream, rowptr, col, val, ix.split, x, ix.zpart, m, d,
                           ix.Wc);
        mk(K_GRAD_MAIN);
        hipLaunchKernelGGL(csr_atr_kernel, grid, block, lds_bytes, stream, rowptr, col, val, y, ix.zpart, ix.split, x,
                           grad, m, d, ix.R, ix.Wc, lambda);
        mk(K_GRAD_MAIN);
        return hipGetLastError();
    }
    int64_t rb = (d + kThreads - 1) / kThreads;
    if (rb > 1024) rb = 1024;
    hipLaunchKernelGGL(csr_regulariser_kernel, dim3((unsigned)rb, (unsigned)n), dim3(kThreads), 0, stream, x, grad, d,
                       lambda);
    mk(K_GRAD_AUX);
    hipLaunchKernelGGL(csr_atomic_kernel, dim3(row_blocks(rows)), dim3(kThreads), 0, stream, rowptr, col, val, y, x,
                       grad, rows, m, d, 1.0f / (float)m);
    mk(K_GRAD_MAIN);
    return hipGetLastError();
}

}  // namespace ef21
