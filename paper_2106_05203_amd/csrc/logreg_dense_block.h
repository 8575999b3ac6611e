// The one-pass dense gradient of eq. (9) as device code shared by the kernels that run it (the gradient kernel
// and the fused small-problem iteration), so that both produce the same bits: the plan that cuts a worker's
// rows into blocks, and the work of one block of kDenseWaves wavefronts.
#pragma once
#include "device_utils.h"

namespace ef21 {

constexpr int kDenseThreads = 256;                    // threads of one row block
constexpr int kDenseWaves = kDenseThreads / kWave;

struct DensePlan {
    int64_t rows_per_wg;
    int64_t chunks;   // row blocks per worker
};

// About two workgroups per compute unit in all (512 on 256 CUs), each streaming one long block of rows:
// fewer, longer blocks measured faster than several rounds of short ones, and they leave fewer partial
// sums to add.  At least 8 rows each.
inline DensePlan dense_plan(int32_t n, int64_t m) {
    int64_t target = 512 / n;
    if (target < 1) target = 1;
    int64_t rows = (m + target - 1) / target;
    if (rows < 8) rows = 8;
    return {rows, (m + rows - 1) / rows};
}

// No batch of tau <= m rows gets more blocks per worker than this (the partial sums are sized by it).
inline int64_t max_chunks(int32_t n, int64_t m) {
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

// One row block: rows [chunk * rows_per_wg, +rows_per_wg) of `worker`, by kDenseWaves wavefronts (`wave` = this
// wavefront's number among them, `tid` = the thread's among their kDenseThreads).  A wavefront owns whole rows;
// a lane keeps its columns of the row in registers between the dot product (wavefront reduction) and the
// rank-one accumulation coef * a_l.  `red` (NQ * kWave * VEC floats of LDS, the block's own) adds the
// wavefronts' accumulators in wavefront order; the result goes to part[worker][chunk][0..d).  Every thread of
// the workgroup must call (it holds workgroup barriers); `active` = false does no work and writes nothing.
// BATCH: the m rows of a worker are the entries of batch[worker][0..m) (row numbers inside its m_full rows), the
// minibatch of Algorithm 5; otherwise m_full == m and row l is row l.
template <int VEC, int NQ, int ROWS, bool BATCH>
__device__ __forceinline__ void dense_block(const float *__restrict__ A, const float *__restrict__ y,
                                            const float *__restrict__ x, float *__restrict__ part, int64_t m,
                                            int64_t d, int64_t rows_per_wg, int loss,
                                            const int32_t *__restrict__ batch, int64_t m_full, int64_t worker,
                                            int64_t chunk, int64_t chunks, int wave, int tid, bool active,
                                            float *red) {
    constexpr int kCols = NQ * kWave * VEC;   // columns covered by one wavefront
    const int lane = lane_id();

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
    const int64_t l1 = !active ? l0 : (l0 + rows_per_wg < m ? l0 + rows_per_wg : m);
    for (int64_t l = l0 + wave * ROWS; l < l1; l += kDenseWaves * ROWS) {
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

    // add the wavefronts' accumulators in wavefront order
    for (int w = 0; w < kDenseWaves; ++w) {
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
    if (active) {
        float *out = part + (worker * chunks + chunk) * d;
        for (int c = tid; c < kCols && c < d; c += kDenseThreads) out[c] = red[c];
    }
}

// Which instantiation (VEC, NQ) of dense_block serves rows of d columns: the kernels that must agree bit for
// bit choose through this one function.  vec4: d % 4 == 0 and A 16-byte aligned.  {0, 0}: none (two passes).
struct DenseVariant {
    int vec, nq;
};
inline DenseVariant dense_variant(int64_t d, bool vec4) {
    if (vec4 && d <= 256) return {4, 1};
    if (vec4 && d <= 512) return {4, 2};
    if (vec4 && d <= 1024) return {4, 4};
    if (vec4 && d <= 2048) return {4, 8};
    if (vec4 && d <= 4096) return {4, 16};
    if (d <= 128) return {1, 2};
    if (d <= 512) return {1, 8};
    if (d <= 2048) return {1, 32};
    return {0, 0};
}

// Rows of a wavefront in flight: 32 row entries per lane for narrow rows (a wavefront would otherwise have only
// a kilobyte or two of loads outstanding; more does not fit the registers of the 1024-thread kernel that shares
// this code), at most eight rows; two rows of 32 entries per lane; one where a row alone fills the registers.
template <int VEC, int NQ>
constexpr int dense_rows_in_flight() {
    constexpr int per_lane = NQ * VEC;
    return per_lane > 32 ? 1 : (per_lane >= 16 ? 2 : (per_lane >= 8 ? 4 : 8));
}

}  // namespace ef21
