// Local gradients of the objective of Section 5, eq. (9), for all workers, sparse (CSR) rows:
//   grad f_i(x) = (1/m) sum_l  -y_l / (1 + exp(y_l a_l^T x)) a_l  +  2 lambda x_j / (1 + x_j^2)^2.
//
// Both halves of this computation are 4-byte random accesses: a gather from x for the dot products and
// a scatter-add into the gradient.  Served from L2 they move a whole cache line per entry and are an
// order of magnitude off the bandwidth roofline; global float atomics are worse still, and LDS float
// atomics are slow too.  So each half is arranged to read a short vector held in LDS and to write
// nothing at random, from its own copy of the matrix.  Needs every row's column indices ascending
// (checked once, when the problem is attached); what is built at attach time, 6 bytes per entry each:
//   - a range-major copy: the columns are cut into R = ceil(d / 12288) ranges; per (range, worker) the
//     rows' slices of that range one after the other, as (16-bit column inside the range, value);
//   - a column-major copy (CSC) of each worker's block: (16-bit row inside the worker, value)
//     (32-bit rows if a worker has more than 65536 of them).
// Per gradient, two streaming passes, both the same segmented sum (segment_sums below):
//   pass 1  segments = row slices, vector = the range of x in LDS: partial dot products z_part[range][row]
//   coef    coef_l = r_l / m from the summed partial dot products (one thread per row)
//   pass 2  segments = columns, vector = the worker's coef (m floats) in LDS: the gradient entries,
//           plus the regulariser term
// No atomics; every sum is taken in a fixed order (bitwise reproducible).
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
constexpr int kCscGroups = 4;         // groups of 64 consecutive columns per wavefront
constexpr int kCscCols = kCscWaves * kCscGroups * kWave;   // columns per workgroup
constexpr int kTile = 1024;           // staged products per wavefront: four loads of four entries per lane
constexpr int64_t kCscPad = 2048;     // zeroed entries after the column-major copy (tiles are loaded whole)
constexpr int64_t kIdx16Rows = 65536; // m up to this: 16-bit row indices in the column-major copy
constexpr int kLongColumn = 128;      // a longer piece of a segment inside one tile is summed by the whole wavefront
constexpr int64_t kCoefLdsRows = 16384;   // m up to this: coef vector in LDS (64 KB)
constexpr int kRangeCols = 12288;     // at most this many columns per range (48 KB of LDS as fp32)
constexpr int kMaxRanges = 64;

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
    void *csc_row;      // [nnz + kCscPad] row inside the worker: uint16 if m <= kIdx16Rows, else int32
    float *csc_val;     // [nnz + kCscPad]
    int64_t *bstart;    // [R][n] first entry of the (range, worker) block of the range-major copy
    int32_t *rptr;      // [R][n][m + 1] start of each row's slice inside its block
    uint16_t *rcol;     // [nnz + kCscPad] column minus the range's first column
    float *rval;        // [nnz + kCscPad]
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
    char *cr = take((m <= kIdx16Rows ? sizeof(uint16_t) : sizeof(int32_t)) * (size_t)(nnz + kCscPad));
    char *cv = take(sizeof(float) * (size_t)(nnz + kCscPad));
    char *bs = take(sizeof(int64_t) * (size_t)R * n);
    char *rp = take(sizeof(int32_t) * (size_t)R * n * (m + 1));
    char *rc = take(sizeof(uint16_t) * (size_t)(nnz + kCscPad));
    char *rv = take(sizeof(float) * (size_t)(nnz + kCscPad));
    if (out) {
        out->bad = (uint32_t *)b;
        out->zpart = (float *)c;
        out->split = (int32_t *)s;
        out->coef = (float *)cf;
        out->colptr = (int32_t *)cp;
        out->csc_row = (void *)cr;
        out->csc_val = (float *)cv;
        out->bstart = (int64_t *)bs;
        out->rptr = (int32_t *)rp;
        out->rcol = (uint16_t *)rc;
        out->rval = (float *)rv;
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

// The fill of the column-major copy walks a worker's rows kRows at a time: lanes 0..kRows-1 fetch the
// bounds of the rows' slices (split is [R + 1][rows]), the bounds are broadcast, and the slices' loads are
// issued for all kRows rows before anything is consumed.  Addresses past a slice's end are clamped to
// its last entry and their contribution dropped, so that no load sits behind a branch.
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

// ---- attach time: the range-major copy.  One workgroup per (range, worker): where the block starts,
// where each row's slice starts inside it, then the slices themselves (column minus the range's first).
__global__ __launch_bounds__(kAtrThreads) void csrr_build_kernel(const int64_t *__restrict__ rowptr,
                                                                 const int32_t *__restrict__ col,
                                                                 const float *__restrict__ val,
                                                                 const int32_t *__restrict__ split,
                                                                 int64_t *__restrict__ bstart,
                                                                 int32_t *__restrict__ rptr,
                                                                 uint16_t *__restrict__ rcol,
                                                                 float *__restrict__ rval, int64_t m, int64_t Wc) {
    __shared__ long long part[kAtrWaves];
    __shared__ uint32_t wave_total[kAtrWaves];
    const int range = blockIdx.x;
    const int64_t worker = blockIdx.y, n = gridDim.y, rows = n * m;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    const int32_t *s_lo = split + (int64_t)range * rows + worker * m;
    const int32_t *s_hi = split + (int64_t)(range + 1) * rows + worker * m;
    long long lower = 0;
    for (int64_t l = tid; l < m; l += kAtrThreads) lower += s_lo[l];
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) lower += __shfl_xor(lower, o, kWave);
    if (lane == 0) part[wave] = lower;
    __syncthreads();
    long long base = rowptr[worker * m];
    for (int w = 0; w < kAtrWaves; ++w) base += part[w];
    if (tid == 0) bstart[(int64_t)range * n + worker] = base;
    int32_t *rp = rptr + ((int64_t)range * n + worker) * (m + 1);
    uint32_t carry = 0;
    for (int64_t l0 = 0; l0 < m; l0 += kAtrThreads) {          // exclusive scan of the slice lengths
        const int64_t l = l0 + tid;
        const uint32_t len = l < m ? (uint32_t)(s_hi[l] - s_lo[l]) : 0u;
        const uint32_t incl = wave_inclusive_scan(len);
        __syncthreads();
        if (lane == kWave - 1) wave_total[wave] = incl;
        __syncthreads();
        uint32_t before = carry, all = 0;
        for (int w = 0; w < kAtrWaves; ++w) {
            if (w < wave) before += wave_total[w];
            all += wave_total[w];
        }
        if (l < m) rp[l] = (int32_t)(before + incl - len);
        carry += all;
    }
    if (tid == 0) rp[m] = (int32_t)carry;
    __syncthreads();                                            // rp is read back below
    const int64_t c0 = (int64_t)range * Wc;
    for (int64_t l = wave; l < m; l += kAtrWaves) {
        const int64_t src = rowptr[worker * m + l] + s_lo[l];
        const int32_t len = s_hi[l] - s_lo[l];
        const int64_t before = rp[l];
        for (int32_t t = lane; t < len; t += kWave) {
            rcol[base + before + t] = (uint16_t)(col[src + t] - c0);
            rval[base + before + t] = val[src + t];
        }
    }
}

// ---- both passes: sums over segments of a contiguous list of (index, value) pairs.
// The calling wavefront owns 4 x 64 consecutive segments; lane j holds the entry ranges [b[g], e[g]) of
// segments j, j + 64, ... (ascending and contiguous over (g, lane); an empty range where there is no
// segment).  The span is walked in tiles of 1024 entries aligned to four entries: each lane loads four
// times four consecutive pairs (the next tile's loads are issued before this tile is summed), multiplies the
// values by vec(index) and stages the products in LDS; then every lane adds, for each of its segments, the piece
// that lies in the tile, in storage order (a piece longer than kLongColumn entries by the whole
// wavefront).  acc[g] receives the sums.  The lists must be readable up to three entries past the span.
template <class Index, class VecFn>
__device__ __forceinline__ void segment_sums(const int64_t (&b)[kCscGroups], const int64_t (&e)[kCscGroups],
                                             const Index *__restrict__ index, const float *__restrict__ value,
                                             VecFn vec, float *tile, int lane, float (&acc)[kCscGroups]) {
    const int64_t span_b = __shfl(b[0], 0, kWave), span_e = __shfl(e[kCscGroups - 1], kWave - 1, kWave);
    const int64_t origin = span_b & ~(int64_t)3;               // tiles are aligned to four entries
    // segment bounds and tile positions relative to the origin (a span has fewer than 2^31 entries)
    int32_t rb[kCscGroups], re[kCscGroups];
#pragma unroll
    for (int g = 0; g < kCscGroups; ++g) {
        acc[g] = 0.f;
        rb[g] = (int32_t)(b[g] - origin);
        re[g] = (int32_t)(e[g] - origin);
    }
    const int32_t end = (int32_t)(span_e - origin);
    constexpr int kLoads = kTile / (4 * kWave);                // 4
    const int64_t last4 = (span_e - 1) & ~(int64_t)3;          // last aligned quad that holds an entry of the span
    typedef float v4f __attribute__((ext_vector_type(4)));
    typedef Index v4r __attribute__((ext_vector_type(4)));
    // the loads of a tile: addresses past the span are clamped (they re-read its last quad), so none sits behind
    // a branch
    auto load_tile = [&](int32_t t0, v4r (&r)[kLoads], v4f (&v)[kLoads]) {
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            int64_t at = origin + t0 + u * (4 * kWave) + 4 * lane;
            at = at < last4 ? at : last4;
            r[u] = __builtin_nontemporal_load(reinterpret_cast<const v4r *>(index + at));
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(value + at));
        }
    };
    v4r r[kLoads], r_next[kLoads];
    v4f v[kLoads], v_next[kLoads];
    if (0 < end) load_tile(0, r, v);
    for (int32_t t0 = 0; t0 < end; t0 += kTile) {
        load_tile(t0 + kTile, r_next, v_next);
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            v4f pr;
            pr.x = v[u].x * vec(r[u].x);
            pr.y = v[u].y * vec(r[u].y);
            pr.z = v[u].z * vec(r[u].z);
            pr.w = v[u].w * vec(r[u].w);
            *reinterpret_cast<v4f *>(tile + u * (4 * kWave) + 4 * lane) = pr;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int32_t t1 = t0 + kTile < end ? t0 + kTile : end;
#pragma unroll
        for (int g = 0; g < kCscGroups; ++g) {
            const int32_t lo = (rb[g] > t0 ? rb[g] : t0) - t0, hi = (re[g] < t1 ? re[g] : t1) - t0;   // tile coordinates
            if (__ballot(lo < hi) == 0) continue;              // the group has nothing in this tile (uniform)
            const bool is_long = hi - lo > kLongColumn;
            if (!is_long) {
                int32_t t = lo;
                float a = acc[g];
                for (; t + 4 <= hi; t += 4) a = (((a + tile[t]) + tile[t + 1]) + tile[t + 2]) + tile[t + 3];
                for (; t < hi; ++t) a += tile[t];
                acc[g] = a;
            }
            uint64_t todo = __ballot(is_long);
            while (todo) {                                     // uniform in the wavefront
                const int src = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const int32_t L = __shfl(lo, src, kWave), H = __shfl(hi, src, kWave);
                float part = 0.f;
                for (int32_t t = L + lane; t < H; t += kWave) part += tile[t];
                part = wave_sum(part);
                if (lane == src) acc[g] += part;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            r[u] = r_next[u];
            v[u] = v_next[u];
        }
    }
}

// ---- pass 1: partial dot products from the range-major copy.  Dynamic LDS: Wc floats (the range of x).
// Grid (R * row chunks, n); a workgroup takes kCscCols rows of one (range, worker), a wavefront 256 of them.
__global__ __launch_bounds__(kCscThreads) void csrr_dot_kernel(const int64_t *__restrict__ bstart,
                                                               const int32_t *__restrict__ rptr,
                                                               const uint16_t *__restrict__ rcol,
                                                               const float *__restrict__ rval,
                                                               const float *__restrict__ x, float *__restrict__ zpart,
                                                               int64_t m, int64_t d, int R, int64_t Wc,
                                                               int64_t x_stride) {
    extern __shared__ float x_lds[];
    __shared__ __attribute__((aligned(16))) float tiles[kCscWaves][kTile];
    const int range = blockIdx.x % R;
    const int64_t chunk = blockIdx.x / R, worker = blockIdx.y, n = gridDim.y, rows = n * m;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t c0 = (int64_t)range * Wc;
    const int64_t width = c0 + Wc < d ? Wc : d - c0;
    for (int64_t j = threadIdx.x; j < width; j += kCscThreads) x_lds[j] = x[worker * x_stride + c0 + j];
    __syncthreads();
    const int64_t l_first = (chunk * kCscWaves + wave) * (kCscGroups * kWave);
    if (l_first >= m) return;                                   // the whole wavefront; no barrier follows
    const int64_t base = bstart[(int64_t)range * n + worker];
    const int32_t *rp = rptr + ((int64_t)range * n + worker) * (m + 1);
    int64_t b[kCscGroups], e[kCscGroups];
#pragma unroll
    for (int g = 0; g < kCscGroups; ++g) {
        const int64_t l = l_first + g * kWave + lane;
        b[g] = base + rp[l < m ? l : m];                       // rows past m: an empty range at the end
        e[g] = base + rp[l < m ? l + 1 : m];
    }
    float acc[kCscGroups];
    segment_sums(b, e, rcol, rval, [&](uint16_t c) { return x_lds[c]; }, tiles[wave], lane, acc);
#pragma unroll
    for (int g = 0; g < kCscGroups; ++g) {
        const int64_t l = l_first + g * kWave + lane;
        if (l < m) zpart[(int64_t)range * rows + worker * m + l] = acc[g];
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
template <class RowIndex>
__global__ __launch_bounds__(kWave) void csc_fill_kernel(const int64_t *__restrict__ rowptr,
                                                         const int32_t *__restrict__ col,
                                                         const float *__restrict__ val,
                                                         const int32_t *__restrict__ split,
                                                         const int32_t *__restrict__ colptr,
                                                         RowIndex *__restrict__ csc_row, float *__restrict__ csc_val,
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
                    csc_row[first + pos] = (RowIndex)(l0 + u);
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
                                                            float inv_m, float *__restrict__ coef, int loss) {
    const int64_t row = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (row >= rows) return;
    float z = 0.f;
    for (int r = 0; r < R; ++r) z += zpart[(int64_t)r * rows + row];
    coef[row] = loss_derivative(y[row], z, loss) * inv_m;
}

// ---- pass 2: gradient columns from the column-major copy.  Dynamic LDS: m floats if COEF_LDS.
// A workgroup takes kCscCols columns of one worker, a wavefront 256 of them; vec = the worker's coef.
template <bool COEF_LDS, class RowIndex>
__global__ __launch_bounds__(kCscThreads) void csc_grad_kernel(const int32_t *__restrict__ colptr,
                                                               const RowIndex *__restrict__ csc_row,
                                                               const float *__restrict__ csc_val,
                                                               const int64_t *__restrict__ rowptr,
                                                               const float *__restrict__ coef,
                                                               const float *__restrict__ x, float *__restrict__ grad,
                                                               int64_t m, int64_t d, float lambda, int64_t x_stride) {
    extern __shared__ float coef_lds[];
    __shared__ __attribute__((aligned(16))) float tiles[kCscWaves][kTile];
    const int64_t worker = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const float *cf = coef + worker * m;
    if constexpr (COEF_LDS) {
        for (int64_t l = threadIdx.x; l < m; l += kCscThreads) coef_lds[l] = cf[l];
        __syncthreads();
    }
    const int64_t cb = ((int64_t)blockIdx.x * kCscWaves + wave) * (kCscGroups * kWave);
    if (cb >= d) return;                                        // the whole wavefront; no barrier follows
    const int64_t first = rowptr[worker * m];
    const int32_t *cp = colptr + worker * (d + 1);
    int64_t b[kCscGroups], e[kCscGroups];                      // global entry ranges of this lane's columns
#pragma unroll
    for (int g = 0; g < kCscGroups; ++g) {
        const int64_t c = cb + g * kWave + lane;
        b[g] = first + cp[c < d ? c : d];                      // columns past d: an empty range at the end
        e[g] = first + cp[c < d ? c + 1 : d];
    }
    float acc[kCscGroups];
    segment_sums(b, e, csc_row, csc_val, [&](RowIndex r) { return COEF_LDS ? coef_lds[r] : cf[r]; }, tiles[wave],
                    lane, acc);
#pragma unroll
    for (int g = 0; g < kCscGroups; ++g) {
        const int64_t c = cb + g * kWave + lane;
        if (c < d) grad[worker * d + c] = acc[g] + regulariser_grad(x[worker * x_stride + c], lambda);
    }
}

// ---- fallback: global atomics, any column order
__global__ __launch_bounds__(kThreads) void csr_regulariser_kernel(const float *__restrict__ x,
                                                                   float *__restrict__ grad, int64_t d,
                                                                   float lambda, int64_t x_stride) {
    const int64_t worker = blockIdx.y;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c < d; c += stride)
        grad[worker * d + c] = regulariser_grad(x[worker * x_stride + c], lambda);
}

__global__ __launch_bounds__(kThreads) void csr_atomic_kernel(const int64_t *__restrict__ rowptr,
                                                              const int32_t *__restrict__ col,
                                                              const float *__restrict__ val,
                                                              const float *__restrict__ y,
                                                              const float *__restrict__ x, float *grad, int64_t rows,
                                                              int64_t m, int64_t d, float inv_m, int loss,
                                                              const int32_t *__restrict__ batch, int64_t m_full,
                                                              int64_t x_stride) {
    const int lane = lane_id();
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    // rows = n * m entries; under a batch, entry e of worker e / m names one of that worker's m_full rows
    for (int64_t e = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave; e < rows; e += nwaves) {
        int64_t l = e;
        if (batch) {
            const uint32_t b = (uint32_t)batch[e];
            if (b >= (uint64_t)m_full) continue;        // outside the worker's rows: contributes nothing
            l = (e / m) * m_full + b;
        }
        const int64_t p0 = rowptr[l], p1 = rowptr[l + 1];
        const float *xw = x + (e / m) * x_stride;
        float s = 0.f;
        // a column index outside [0, d) is skipped rather than dereferenced
        for (int64_t p = p0 + lane; p < p1; p += kWave) {
            const uint32_t c = (uint32_t)col[p];
            if (c < (uint64_t)d) s = fmaf(val[p], xw[c], s);
        }
        s = wave_sum(s);
        const float coef = loss_derivative(y[l], s, loss) * inv_m;
        float *g = grad + (e / m) * d;
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
    hipLaunchKernelGGL(csrr_build_kernel, grid, dim3(kAtrThreads), 0, stream, rowptr, col, val, ix.split, ix.bstart,
                       ix.rptr, ix.rcol, ix.rval, m, ix.Wc);
    st = hipMemsetAsync(ix.rcol + nnz, 0, sizeof(uint16_t) * (size_t)kCscPad, stream);
    if (st == hipSuccess) st = hipMemsetAsync(ix.rval + nnz, 0, sizeof(float) * (size_t)kCscPad, stream);
    if (st != hipSuccess) return st;
    const bool idx16 = m <= kIdx16Rows;
    const size_t row_bytes = idx16 ? sizeof(uint16_t) : sizeof(int32_t);
    st = hipMemsetAsync((char *)ix.csc_row + row_bytes * (size_t)nnz, 0, row_bytes * (size_t)kCscPad, stream);
    if (st == hipSuccess) st = hipMemsetAsync(ix.csc_val + nnz, 0, sizeof(float) * (size_t)kCscPad, stream);
    if (st != hipSuccess) return st;
    if (idx16)
        hipLaunchKernelGGL(csc_fill_kernel<uint16_t>, grid, dim3(kWave), lds_bytes, stream, rowptr, col, val, ix.split,
                           ix.colptr, (uint16_t *)ix.csc_row, ix.csc_val, m, d, ix.Wc);
    else
        hipLaunchKernelGGL(csc_fill_kernel<int32_t>, grid, dim3(kWave), lds_bytes, stream, rowptr, col, val, ix.split,
                           ix.colptr, (int32_t *)ix.csc_row, ix.csc_val, m, d, ix.Wc);
    st = hipStreamSynchronize(stream);
    if (st != hipSuccess) return st;
    *usable = true;
    return hipGetLastError();
}

hipError_t launch_logreg_grad_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                                  const float *x, float *grad, int32_t n, int64_t m, int64_t d, int64_t nnz,
                                  float lambda, const void *index, hipStream_t stream, const Marker &mk, int loss,
                                  RowBatch batch, int64_t x_stride) {
    const int32_t *listed = batch.tau > 0 ? batch.rows : nullptr;
    const int64_t rows = (int64_t)n * m;
    if (index && !listed) {
        IndexLayout ix;
        index_layout(n, m, d, nnz, (char *)const_cast<void *>(index), &ix);
        static PerDeviceOnce configured;
        const hipError_t cfg = configured([] {
            hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csrr_dot_kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kRangeCols);
            if (st == hipSuccess)
                st = hipFuncSetAttribute(reinterpret_cast<const void *>(&csc_grad_kernel<true, uint16_t>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, sizeof(float) * kCoefLdsRows);
            return st;
        });
        if (cfg != hipSuccess) return cfg;
        const int64_t row_chunks = (m + kCscCols - 1) / kCscCols;
        hipLaunchKernelGGL(csrr_dot_kernel, dim3((unsigned)(ix.R * row_chunks), (unsigned)n), dim3(kCscThreads),
                           sizeof(float) * (size_t)ix.Wc, stream, ix.bstart, ix.rptr, ix.rcol, ix.rval, x, ix.zpart, m, d,
                           ix.R, ix.Wc, x_stride);
        mk(K_GRAD_MAIN);
        hipLaunchKernelGGL(csr_coef_kernel, dim3((unsigned)((rows + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                           stream, y, ix.zpart, ix.R, rows, 1.0f / (float)m, ix.coef, loss);
        mk(K_GRAD_AUX);
        const dim3 grid((unsigned)((d + kCscCols - 1) / kCscCols), (unsigned)n);
        static_assert(kCoefLdsRows <= kIdx16Rows, "a coefficient vector that fits LDS has 16-bit row indices");
        if (m <= kCoefLdsRows)
            hipLaunchKernelGGL((csc_grad_kernel<true, uint16_t>), grid, dim3(kCscThreads), sizeof(float) * (size_t)m, stream,
                               ix.colptr, (const uint16_t *)ix.csc_row, ix.csc_val, rowptr, ix.coef, x, grad, m, d, lambda, x_stride);
        else if (m <= kIdx16Rows)
            hipLaunchKernelGGL((csc_grad_kernel<false, uint16_t>), grid, dim3(kCscThreads), 0, stream, ix.colptr,
                               (const uint16_t *)ix.csc_row, ix.csc_val, rowptr, ix.coef, x, grad, m, d, lambda, x_stride);
        else
            hipLaunchKernelGGL((csc_grad_kernel<false, int32_t>), grid, dim3(kCscThreads), 0, stream, ix.colptr,
                               (const int32_t *)ix.csc_row, ix.csc_val, rowptr, ix.coef, x, grad, m, d, lambda, x_stride);
        mk(K_GRAD_MAIN);
        return hipGetLastError();
    }
    int64_t rb = (d + kThreads - 1) / kThreads;
    if (rb > 1024) rb = 1024;
    hipLaunchKernelGGL(csr_regulariser_kernel, dim3((unsigned)rb, (unsigned)n), dim3(kThreads), 0, stream, x, grad, d,
                       lambda, x_stride);
    mk(K_GRAD_AUX);
    const int64_t per_worker = listed ? batch.tau : m;
    hipLaunchKernelGGL(csr_atomic_kernel, dim3(row_blocks((int64_t)n * per_worker)), dim3(kThreads), 0, stream, rowptr,
                       col, val, y, x, grad, (int64_t)n * per_worker, per_worker, d, 1.0f / (float)per_worker, loss,
                       listed, m, x_stride);
    mk(K_GRAD_MAIN);
    return hipGetLastError();
}

}  // namespace ef21
