// Local gradients of the objective of Section 5, eq. (9), for all workers, sparse (CSR) rows:
//   grad f_i(x) = (1/m) sum_l  -y_l / (1 + exp(y_l a_l^T x)) a_l  +  2 lambda x_j / (1 + x_j^2)^2.
//
// Both halves of this computation are 4-byte random accesses: a gather from x for the dot products and
// a scatter-add into the gradient.  Served from L2 they move a whole cache line per entry and are an
// order of magnitude off the bandwidth roofline; global float atomics are worse still, and LDS float
// atomics are slow too.  So each half is arranged to read a short vector held in LDS and to write
// nothing at random.  Needs every row's column indices ascending (checked once, when the problem is
// attached); what is built at attach time:
//   - the columns are cut into R = ceil(d / 12288) ranges, and `split` holds where each range starts
//     inside each row, so a range's slice of a row is contiguous;
//   - a column-major copy (CSC) of each worker's block of the matrix: colptr, row index, value.
// Per gradient, two streaming passes over the non-zeros:
//   pass 1 (CSR)  one workgroup per (range, worker), x-range in LDS; one wavefront per row slice:
//                 partial dot product z_part[range][row]
//   coef          coef_l = r_l / m from the summed partial dot products (one thread per row)
//   pass 2 (CSC)  the worker's coef vector (m floats) in LDS; a wavefront owns 64 consecutive columns,
//                 loads their entries coalesced, multiplies by coef[row] and stages the products in LDS,
//                 where every lane sums its own column in storage order -- no atomics, bitwise
//                 reproducible -- and adds the regulariser term
// Unsorted rows, or d too large for the index, fall back to a kernel built on global atomics.
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kAtrThreads = 1024;
constexpr int kAtrWaves = kAtrThreads / kWave;
constexpr int kCscThreads = 512;      // pass 2
constexpr int kCscWaves = kCscThreads / kWave;
constexpr int kCscGroups = 4;         // groups of 64 columns per wavefront
constexpr int kCscCols = kCscWaves * kCscGroups * kWave;   // columns per workgroup
constexpr int kTile = 1024;           // staged products per wavefront
constexpr int kLongColumn = 48;       // a longer piece of a column inside one tile is summed by the whole wavefront
constexpr int64_t kCoefLdsRows = 16384;   // m up to this: coef vector in LDS (64 KB)
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
    float *coef;        // [rows] r_l / m
    int32_t *colptr;    // [n][d + 1] CSC column starts, relative to the worker's first non-zero
    int32_t *csc_row;   // [nnz] row inside the worker
    float *csc_val;     // [nnz]
    int R;
    int64_t Wc;
};

size_t index_layout(int32_t n, int64_t m, int64_t d, int64_t nnz, char *base, IndexLayout *out) {
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
    char *cf = take(sizeof(float) * (size_t)rows);
    char *cp = take(sizeof(int32_t) * (size_t)n * (d + 1));
    char *cr = take(sizeof(int32_t) * (size_t)nnz);
    char *cv = take(sizeof(float) * (size_t)nnz);
    if (out) {
        out->bad = (uint32_t *)b;
        out->zpart = (float *)c;
        out->split = (int32_t *)s;
        out->coef = (float *)cf;
        out->colptr = (int32_t *)cp;
        out->csc_row = (int32_t *)cr;
        out->csc_val = (float *)cv;
        out->R = (int)R;
        out->Wc = Wc;
    }
    return off;
}

bool index_possible(int64_t d) { return (d + kRangeCols - 1) / kRangeCols <= kMaxRanges; }

// ---- attach time
__global__ __launch_bounds__(kThreads) void csr_inspect_kernel(const int64_t *__restrict__ rowptr,
                                                               const int32_t *__restrict__ col, int64_t rows,
                                                               int64_t m, int64_t d, uint32_t *bad) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t l = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; l < rows; l += nwaves) {
        const int64_t p0 = rowptr[l], p1 = rowptr[l + 1];
        bool wrong = p1 < p0 || p1 - p0 > 0x7fffffff;
        // the CSC offsets of a worker are int32
        if (l % m == 0 && rowptr[l + m] - p0 > 0x7fff0000) wrong = true;
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

// ---- attach time: the column-major copy.
// Column starts of one (range, worker): counts in LDS, exclusive scan, plus the number of the worker's
// entries in lower ranges.  Dynamic LDS: Wc words.
__global__ __launch_bounds__(kAtrThreads) void csc_count_kernel(const int64_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ col,
                                                                const int32_t *__restrict__ split,
                                                                int32_t *__restrict__ colptr, int64_t m, int64_t d,
                                                                int R, int64_t Wc) {
    extern __shared__ uint32_t cnt[];
    __shared__ uint32_t wave_total[kAtrWaves];
    __shared__ long long lower_part[kAtrWaves];
    const int range = blockIdx.x;
    const int64_t worker = blockIdx.y, rows = (int64_t)gridDim.y * m;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    const int64_t c0 = (int64_t)range * Wc;
    const int64_t width = c0 + Wc < d ? Wc : (d > c0 ? d - c0 : 0);
    for (int64_t j = tid; j < Wc; j += kAtrThreads) cnt[j] = 0u;
    __syncthreads();
    for (int64_t l = wave; l < m; l += kAtrWaves) {
        const int64_t row = worker * m + l;
        const int64_t p0 = rowptr[row] + split[(int64_t)range * rows + row];
        const int64_t p1 = rowptr[row] + split[(int64_t)(range + 1) * rows + row];
        for (int64_t p = p0 + lane; p < p1; p += kWave) atomicAdd(&cnt[col[p] - c0], 1u);
    }
    // the worker's entries in lower ranges: sum over its rows of where this range starts in the row
    long long lower = 0;
    for (int64_t l = tid; l < m; l += kAtrThreads) lower += split[(int64_t)range * rows + worker * m + l];
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) lower += __shfl_xor(lower, o, kWave);
    if (lane == 0) lower_part[wave] = lower;
    __syncthreads();

    constexpr int kPer = kRangeCols / kAtrThreads;     // consecutive columns per thread
    uint32_t before[kPer], mine = 0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int64_t j = (int64_t)tid * kPer + q;
        before[q] = mine;
        mine += j < width ? cnt[j] : 0u;
    }
    const uint32_t incl = wave_inclusive_scan(mine);
    if (lane == kWave - 1) wave_total[wave] = incl;
    __syncthreads();
    long long base = 0;
    for (int w = 0; w < kAtrWaves; ++w) base += lower_part[w];
    uint32_t start = incl - mine;
    for (int w = 0; w < wave; ++w) start += wave_total[w];
    int32_t *out = colptr + worker * (d + 1) + c0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int64_t j = (int64_t)tid * kPer + q;
        if (j < width) out[j] = (int32_t)(base + start + before[q]);
    }
    if (range == R - 1 && tid == 0)
        colptr[worker * (d + 1) + d] = (int32_t)(rowptr[(worker + 1) * m] - rowptr[worker * m]);
}

// Entries of one (range, worker) into their columns.  ONE wavefront walks the worker's rows in a fixed
// order and hands out the positions inside each column from a cursor in LDS (the columns of a row are
// distinct, so the lanes of one step never meet), which makes the order inside a column -- hence the
// order of the floating-point sums of pass 2 -- a function of the matrix alone.  Dynamic LDS: Wc words.
__global__ __launch_bounds__(kWave) void csc_fill_kernel(const int64_t *__restrict__ rowptr,
                                                         const int32_t *__restrict__ col,
                                                         const float *__restrict__ val,
                                                         const int32_t *__restrict__ split,
                                                         const int32_t *__restrict__ colptr,
                                                         int32_t *__restrict__ csc_row, float *__restrict__ csc_val,
                                                         int64_t m, int64_t d, int64_t Wc) {
    extern __shared__ uint32_t cursor[];
    const int range = blockIdx.x;
    const int64_t worker = blockIdx.y, rows = (int64_t)gridDim.y * m;
    const int lane = lane_id();
    const int64_t c0 = (int64_t)range * Wc;
    const int64_t width = c0 + Wc < d ? Wc : (d > c0 ? d - c0 : 0);
    for (int64_t j = lane; j < width; j += kWave) cursor[j] = (uint32_t)colptr[worker * (d + 1) + c0 + j];
    __syncthreads();
    const int64_t first = rowptr[worker * m];
    for (int64_t l0 = 0; l0 < m; l0 += kRows) {
        const SliceBounds mine = batch_bounds(rowptr, split, rows, range, worker, m, l0, lane);
        const int32_t longest = batch_longest(mine.len);
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
                c[u] = len > 0 ? col[at] : (int32_t)c0;
                v[u] = len > 0 ? val[at] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                if (in[u]) {
                    const uint32_t pos = cursor[c[u] - c0];
                    cursor[c[u] - c0] = pos + 1u;
                    csc_row[first + pos] = (int32_t)(l0 + u);
                    csc_val[first + pos] = v[u];
                }
            }
        }
    }
}

// ---- coef_l = r_l / m with r_l the derivative of the logistic term at z_l = sum of the partial dot
// products (added in range order)
__global__ __launch_bounds__(kThreads) void csr_coef_kernel(const float *__restrict__ y,
                                                            const float *__restrict__ zpart, int R, int64_t rows,
                                                            float inv_m, float *__restrict__ coef) {
    const int64_t row = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (row >= rows) return;
    float z = 0.f;
    for (int r = 0; r < R; ++r) z += zpart[(int64_t)r * rows + row];
    coef[row] = residual(y[row], z) * inv_m;
}

// ---- pass 2: gradient columns from the column-major copy.  Dynamic LDS: m floats if COEF_LDS.
template <bool COEF_LDS>
__global__ __launch_bounds__(kCscThreads) void csc_grad_kernel(const int32_t *__restrict__ colptr,
                                                               const int32_t *__restrict__ csc_row,
                                                               const float *__restrict__ csc_val,
                                                               const int64_t *__restrict__ rowptr,
                                                               const float *__restrict__ coef,
                                                               const float *__restrict__ x, float *__restrict__ grad,
                                                               int64_t m, int64_t d, float lambda) {
    extern __shared__ float coef_lds[];
    __shared__ float tiles[kCscWaves][kTile];
    const int64_t worker = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const float *cf = coef + worker * m;
    if constexpr (COEF_LDS) {
        for (int64_t l = threadIdx.x; l < m; l += kCscThreads) coef_lds[l] = cf[l];
        __syncthreads();
    }
    const int64_t first = rowptr[worker * m];
    const int32_t *rw = csc_row + first;
    const float *vl = csc_val + first;
    const int32_t *cp = colptr + worker * (d + 1);
    float *tile = tiles[wave];

    for (int g = 0; g < kCscGroups; ++g) {
        const int64_t cb = ((int64_t)blockIdx.x * kCscGroups + g) * (kCscWaves * kWave) + wave * kWave;
        if (cb >= d) break;                                    // uniform in the wavefront
        const bool has_col = cb + lane < d;                    // lanes past d hold an empty piece at the end
        const int32_t b = cp[has_col ? cb + lane : d], e = cp[has_col ? cb + lane + 1 : d];
        const int32_t B = __shfl(b, 0, kWave), E = __shfl(e, kWave - 1, kWave);
        float acc = 0.f;
        for (int32_t t0 = B; t0 < E; t0 += kTile) {
            // stage the products of up to kTile entries, 256 at a time, all loads of a block in flight
            constexpr int kUnroll = 4;
            for (int32_t s0 = 0; s0 < kTile && t0 + s0 < E; s0 += kUnroll * kWave) {
                int32_t r[kUnroll];
                float v[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int32_t t = t0 + s0 + u * kWave + lane;
                    const int32_t at = t < E ? t : E - 1;       // clamped: no load behind a branch
                    r[u] = stream_load(rw + at);
                    v[u] = stream_load(vl + at);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const float c = COEF_LDS ? coef_lds[r[u]] : cf[r[u]];
                    tile[s0 + u * kWave + lane] = v[u] * c;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // every lane adds the piece of its column that lies in this tile, in storage order
            const int32_t t1 = t0 + kTile < E ? t0 + kTile : E;
            const int32_t lo = b > t0 ? b : t0, hi = e < t1 ? e : t1;
            const bool is_long = hi - lo > kLongColumn;
            if (!is_long)
                for (int32_t t = lo; t < hi; ++t) acc += tile[t - t0];
            uint64_t todo = __ballot(is_long);
            while (todo) {                                       // uniform in the wavefront
                const int src = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const int32_t L = __shfl(lo, src, kWave), H = __shfl(hi, src, kWave);
                float part = 0.f;
                for (int32_t t = L + lane; t < H; t += kWave) part += tile[t - t0];
                part = wave_sum(part);
                if (lane == src) acc += part;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (cb + lane < d) grad[worker * d + cb + lane] = acc + regulariser_grad(x[cb + lane], lambda);
    }
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

size_t logreg_csr_index_bytes(int32_t n, int64_t m, int64_t d, int64_t nnz) {
    return index_possible(d) ? index_layout(n, m, d, nnz, nullptr, nullptr) : 0;
}

hipError_t logreg_csr_build_index(const int64_t *rowptr, const int32_t *col, const float *val, int32_t n, int64_t m,
                                  int64_t d, int64_t nnz, void *index, hipStream_t stream, bool *usable) {
    *usable = false;
    if (!index || !index_possible(d)) return hipSuccess;
    IndexLayout ix;
    index_layout(n, m, d, nnz, (char *)index, &ix);
    const int64_t rows = (int64_t)n * m;
    hipError_t st = hipMemsetAsync(ix.bad, 0, 256, stream);
    if (st != hipSuccess) return st;
    hipLaunchKernelGGL(csr_inspect_kernel, dim3(row_blocks(rows)), dim3(kThreads), 0, stream, rowptr, col, rows, m, d,
                       ix.bad);
    uint32_t bad = 0;
    st = hipMemcpyAsync(&bad, ix.bad, sizeof(bad), hipMemcpyDeviceToHost, stream);
    if (st != hipSuccess) return st;
    st = hipStreamSynchronize(stream);
    if (st != hipSuccess) return st;
    if (bad != 0) return hipSuccess;      // not ascending everywhere: the caller uses the atomic kernel
    hipLaunchKernelGGL(csr_split_kernel, dim3(row_blocks(rows)), dim3(kThreads), 0, stream, rowptr, col, rows, ix.R,
                       ix.Wc, ix.split);
    const dim3 grid((unsigned)ix.R, (unsigned)n);
    const size_t lds_bytes = sizeof(uint32_t) * (size_t)ix.Wc;
    hipLaunchKernelGGL(csc_count_kernel, grid, dim3(kAtrThreads), lds_bytes, stream, rowptr, col, ix.split, ix.colptr,
                       m, d, ix.R, ix.Wc);
    hipLaunchKernelGGL(csc_fill_kernel, grid, dim3(kWave), lds_bytes, stream, rowptr, col, val, ix.split, ix.colptr,
                       ix.csc_row, ix.csc_val, m, d, ix.Wc);
    st = hipStreamSynchronize(stream);
    if (st != hipSuccess) return st;
    *usable = true;
    return hipGetLastError();
}

hipError_t launch_logreg_grad_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                                  const float *x, float *grad, int32_t n, int64_t m, int64_t d, int64_t nnz,
                                  float lambda, const void *index, hipStream_t stream, const Marker &mk) {
    const int64_t rows = (int64_t)n * m;
    if (index) {
        IndexLayout ix;
        index_layout(n, m, d, nnz, (char *)const_cast<void *>(index), &ix);
        static bool configured = false;
        if (!configured) {
            hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csr_dot_kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kRangeCols);
            if (st == hipSuccess)
                st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csc_grad_kernel<true>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kCoefLdsRows);
            if (st != hipSuccess) return st;
            configured = true;
        }
        hipLaunchKernelGGL(csr_dot_kernel, dim3((unsigned)ix.R, (unsigned)n), dim3(kAtrThreads),
                           sizeof(float) * (size_t)ix.Wc, stream, rowptr, col, val, ix.split, x, ix.zpart, m, d, ix.Wc);
        mk(K_GRAD_MAIN);
        hipLaunchKernelGGL(csr_coef_kernel, dim3((unsigned)((rows + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                           stream, y, ix.zpart, ix.R, rows, 1.0f / (float)m, ix.coef);
        mk(K_GRAD_AUX);
        const dim3 grid((unsigned)((d + kCscCols - 1) / kCscCols), (unsigned)n);
        if (m <= kCoefLdsRows)
            hipLaunchKernelGGL(csc_grad_kernel<true>, grid, dim3(kCscThreads), sizeof(float) * (size_t)m, stream,
                               ix.colptr, ix.csc_row, ix.csc_val, rowptr, ix.coef, x, grad, m, d, lambda);
        else
            hipLaunchKernelGGL(csc_grad_kernel<false>, grid, dim3(kCscThreads), 0, stream, ix.colptr, ix.csc_row,
                               ix.csc_val, rowptr, ix.coef, x, grad, m, d, lambda);
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
