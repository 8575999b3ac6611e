// EF21+ (Algorithm 3 of the EF21 paper): per worker, the better of the plain compressor b = C(s) and the
// Markov compressor m = g_i + C(s - g_i), s = grad f_i(x), C = Top-k.  The two Top-k selections are the
// library's ordinary ones; this file holds what is particular to Algorithm 3:
//   line 7  the distortions B = ||b - s||^2 = ||s||^2 - sum of the kept s_j^2 and
//           M = ||m - s||^2 = ||s - g_i||^2 - sum of the kept (s_j - g_ij)^2 (at a kept position m_j equals s_j
//           up to the rounding of one fp32 addition), differences and sums in fp64, in a fixed order;
//   line 8  g_i <- m if M <= B, else b: a sparse update, or a rewrite of the whole row;
//   line 10 g = (1/n) sum_i g_i is then recomputed from the rows (launch_mean_rows).
#include <algorithm>

#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int64_t kNormChunk = 1 << 16;      // entries of a row per workgroup of the norm / rewrite kernels

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum over the workgroup, the same value in every thread; `lds` holds kWaves doubles.
__device__ double block_sum_f64(double v, double *lds) {
    v = wave_sum_f64(v);
    __syncthreads();                       // lds may still be read from a previous call
    if (lane_id() == 0) lds[threadIdx.x / kWave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < kWaves; ++w) t += lds[w];
    return t;
}

// part[row][chunk] = (sum s^2, sum (s - g_i)^2) over the chunk, the differences of the stored values taken
// exactly (in fp64), as the distortions of line 7 are defined on the stored vectors.  VEC = 4 (rows of a
// multiple of four entries, 16-byte aligned): four float4 loads per array in flight per thread.
template <int VEC>
__global__ __launch_bounds__(kThreads) void plus_sqnorms_kernel(const float *__restrict__ s,
                                                                const float *__restrict__ g_i, int64_t d,
                                                                double2 *__restrict__ part) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.y, chunk = blockIdx.x;
    const int64_t lo = chunk * kNormChunk, hi = lo + kNormChunk < d ? lo + kNormChunk : d;
    const float *sr = s + row * d, *gr = g_i + row * d;
    double acc_s = 0.0, acc_v = 0.0;
    if constexpr (VEC == 4) {
        constexpr int kUnroll = 4;
        constexpr int64_t kStep = (int64_t)kThreads * 4;
        int64_t e = lo + (int64_t)threadIdx.x * 4;
        for (; e + (kUnroll - 1) * kStep + 4 <= hi; e += kUnroll * kStep) {
            float4 a[kUnroll], b[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                a[u] = stream_load4(sr + e + u * kStep);
                b[u] = stream_load4(gr + e + u * kStep);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const double s0 = a[u].x, s1 = a[u].y, s2 = a[u].z, s3 = a[u].w;
                const double v0 = s0 - (double)b[u].x, v1 = s1 - (double)b[u].y, v2 = s2 - (double)b[u].z,
                             v3 = s3 - (double)b[u].w;                       // exact
                acc_s += (s0 * s0 + s1 * s1) + (s2 * s2 + s3 * s3);
                acc_v += (v0 * v0 + v1 * v1) + (v2 * v2 + v3 * v3);
            }
        }
        for (; e + 4 <= hi; e += kStep) {
            const float4 a = stream_load4(sr + e), b = stream_load4(gr + e);
            const double s0 = a.x, s1 = a.y, s2 = a.z, s3 = a.w;
            const double v0 = s0 - (double)b.x, v1 = s1 - (double)b.y, v2 = s2 - (double)b.z, v3 = s3 - (double)b.w;
            acc_s += (s0 * s0 + s1 * s1) + (s2 * s2 + s3 * s3);
            acc_v += (v0 * v0 + v1 * v1) + (v2 * v2 + v3 * v3);
        }
    } else {
        for (int64_t e = lo + threadIdx.x; e < hi; e += kThreads) {
            const double sv = (double)stream_load(sr + e), v = sv - (double)stream_load(gr + e);   // exact
            acc_s += sv * sv;
            acc_v += v * v;
        }
    }
    acc_s = block_sum_f64(acc_s, lds);
    acc_v = block_sum_f64(acc_v, lds);
    if (threadIdx.x == 0) part[row * gridDim.x + chunk] = make_double2(acc_s, acc_v);
}

// What the kept entries take away from the two norms, per block of kKeptBlock message entries:
// kept[row][blk] = (sum of b_j^2, sum of (s_j - g_ij)^2 over the positions of m).  b_j = s_j exactly; m_j = s_j
// up to the rounding of the fp32 update, so the exact (s_j - g_ij)^2 leaves the sum.
constexpr int64_t kKeptBlock = (int64_t)kThreads * 8;

__global__ __launch_bounds__(kThreads) void plus_kept_kernel(const float *__restrict__ s,
                                                             const float *__restrict__ g_i, int64_t d,
                                                             const float *__restrict__ val_b,
                                                             const int32_t *__restrict__ idx_m, int64_t k,
                                                             double2 *__restrict__ kept) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.y;
    const int64_t lo = (int64_t)blockIdx.x * kKeptBlock, hi = lo + kKeptBlock < k ? lo + kKeptBlock : k;
    double kb = 0.0, km = 0.0;
    for (int64_t j = lo + threadIdx.x; j < hi; j += kThreads) {
        const double vb = (double)val_b[row * k + j];
        const int64_t e = idx_m[row * k + j];
        const double vm = (double)s[row * d + e] - (double)g_i[row * d + e];
        kb += vb * vb;
        km += vm * vm;
    }
    kb = block_sum_f64(kb, lds);
    km = block_sum_f64(km, lds);
    if (threadIdx.x == 0) kept[row * gridDim.x + blockIdx.x] = make_double2(kb, km);
}

// One workgroup per worker: B, M and the choice of line 8 from the partial sums (each added in a fixed order).
// kblocks == 0 (short messages): the kept sums are taken here, from the messages themselves.
__global__ __launch_bounds__(kThreads) void plus_decide_kernel(const double2 *__restrict__ part, int64_t chunks,
                                                               const double2 *__restrict__ kept, int64_t kblocks,
                                                               const float *__restrict__ s,
                                                               const float *__restrict__ g_i, int64_t d,
                                                               const float *__restrict__ val_b,
                                                               const int32_t *__restrict__ idx_m, int64_t k,
                                                               int32_t *__restrict__ branch, double *__restrict__ BM) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.x;
    double ns = 0.0, nv = 0.0, kb = 0.0, km = 0.0;
    for (int64_t c = threadIdx.x; c < chunks; c += kThreads) {
        const double2 p = part[row * chunks + c];
        ns += p.x;
        nv += p.y;
    }
    for (int64_t c = threadIdx.x; c < kblocks; c += kThreads) {
        const double2 p = kept[row * kblocks + c];
        kb += p.x;
        km += p.y;
    }
    if (kblocks == 0) {
        for (int64_t j = threadIdx.x; j < k; j += kThreads) {
            const double vb = (double)val_b[row * k + j];
            const int64_t e = idx_m[row * k + j];
            const double vm = (double)s[row * d + e] - (double)g_i[row * d + e];
            kb += vb * vb;
            km += vm * vm;
        }
    }
    ns = block_sum_f64(ns, lds);
    nv = block_sum_f64(nv, lds);
    kb = block_sum_f64(kb, lds);
    km = block_sum_f64(km, lds);
    const double B = ns - kb, M = nv - km;
    if (threadIdx.x == 0) {
        branch[row] = M > B ? 1 : 0;                // line 8: the Markov compressor unless it is strictly worse
        BM[2 * row] = B;
        BM[2 * row + 1] = M;
    }
}

// Rows whose worker chose the plain compressor are cleared (g_i <- b has k non-zeros at most).
template <int VEC>
__global__ __launch_bounds__(kThreads) void plus_clear_kernel(const int32_t *__restrict__ branch,
                                                              float *__restrict__ g_i, int64_t d) {
    const int64_t row = blockIdx.y;
    if (!branch[row]) return;
    const int64_t lo = (int64_t)blockIdx.x * kNormChunk, hi = lo + kNormChunk < d ? lo + kNormChunk : d;
    float *gr = g_i + row * d;
    if constexpr (VEC == 4) {
        for (int64_t e = lo + (int64_t)threadIdx.x * 4; e + 4 <= hi; e += (int64_t)kThreads * 4)
            *reinterpret_cast<float4 *>(gr + e) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        for (int64_t e = lo + threadIdx.x; e < hi; e += kThreads) gr[e] = 0.f;
    }
}

// The k entries of the chosen message, copied to (msg_idx, msg_val) and applied: added to g_i (Markov branch,
// one fp32 addition each) or written into the cleared row (plain branch).
__global__ __launch_bounds__(kThreads) void plus_apply_kernel(const int32_t *__restrict__ branch,
                                                              const int32_t *__restrict__ idx_b,
                                                              const float *__restrict__ val_b,
                                                              const int32_t *__restrict__ idx_m,
                                                              const float *__restrict__ val_m, int64_t k,
                                                              int32_t *__restrict__ msg_idx,
                                                              float *__restrict__ msg_val, float *__restrict__ g_i,
                                                              int64_t d) {
    const int64_t row = blockIdx.y;
    const bool plain = branch[row] != 0;
    const int32_t *ci = plain ? idx_b : idx_m;
    const float *cv = plain ? val_b : val_m;
    float *gr = g_i + row * d;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < k; j += stride) {
        const int32_t e = ci[row * k + j];
        const float v = cv[row * k + j];
        msg_idx[row * k + j] = e;
        msg_val[row * k + j] = v;
        gr[e] = plain ? v : gr[e] + v;
    }
}

int64_t chunks_of(int64_t d) { return (d + kNormChunk - 1) / kNormChunk; }
int64_t kept_blocks_of(int64_t k) { return (k + kKeptBlock - 1) / kKeptBlock; }

}  // namespace

// room for the norm partials of either producer: the norm kernel's chunks, or one per piece of the long-row Top-k
int64_t plus_norm_chunks_max(int32_t n, int64_t d) { return std::max<int64_t>(chunks_of(d), topk_split_slots(n, d)); }

size_t plus_scratch_bytes(int32_t n, int64_t d, int64_t k) {
    return sizeof(double2) * (size_t)n * (size_t)(plus_norm_chunks_max(n, d) + kept_blocks_of(k));
}

hipError_t launch_plus_choose(const float *s, float *g_i, int32_t n, int64_t d, int64_t k, const int32_t *idx_b,
                              const float *val_b, const int32_t *idx_m, const float *val_m, void *scratch,
                              int32_t *branch, double *BM, int32_t *msg_idx, float *msg_val, hipStream_t stream,
                              int64_t norm_chunks) {
    if (norm_chunks < 0 || norm_chunks > plus_norm_chunks_max(n, d)) return hipErrorInvalidValue;
    const int64_t chunks = norm_chunks > 0 ? norm_chunks : chunks_of(d), grid_chunks = chunks_of(d);
    double2 *part = (double2 *)scratch;
    // kNormChunk is a multiple of four, so with d % 4 == 0 every chunk is whole float4s
    const bool vec4 = (d % 4 == 0) && (((uintptr_t)s | (uintptr_t)g_i) % 16 == 0);
    if (norm_chunks > 0) {
        // the partial sums are already there
    } else if (vec4) {
        hipLaunchKernelGGL(plus_sqnorms_kernel<4>, dim3((unsigned)chunks, (unsigned)n), dim3(kThreads), 0, stream, s,
                           g_i, d, part);
    } else {
        hipLaunchKernelGGL(plus_sqnorms_kernel<1>, dim3((unsigned)chunks, (unsigned)n), dim3(kThreads), 0, stream, s,
                           g_i, d, part);
    }
    const int64_t kblocks = k <= kKeptBlock ? 0 : kept_blocks_of(k);     // short messages: summed by the decide kernel
    double2 *kept = part + (size_t)n * plus_norm_chunks_max(n, d);
    if (kblocks > 0)
        hipLaunchKernelGGL(plus_kept_kernel, dim3((unsigned)kblocks, (unsigned)n), dim3(kThreads), 0, stream, s, g_i,
                           d, val_b, idx_m, k, kept);
    hipLaunchKernelGGL(plus_decide_kernel, dim3((unsigned)n), dim3(kThreads), 0, stream, part, chunks, kept, kblocks, s,
                       g_i, d, val_b, idx_m, k, branch, BM);
    if (vec4)
        hipLaunchKernelGGL(plus_clear_kernel<4>, dim3((unsigned)grid_chunks, (unsigned)n), dim3(kThreads), 0, stream,
                           branch, g_i, d);
    else
        hipLaunchKernelGGL(plus_clear_kernel<1>, dim3((unsigned)grid_chunks, (unsigned)n), dim3(kThreads), 0, stream,
                           branch, g_i, d);
    int64_t blocks = (k + kThreads - 1) / kThreads;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(plus_apply_kernel, dim3((unsigned)blocks, (unsigned)n), dim3(kThreads), 0, stream, branch,
                       idx_b, val_b, idx_m, val_m, k, msg_idx, msg_val, g_i, d);
    return hipGetLastError();
}

}  // namespace ef21
