// EF21+ (Algorithm 3 of the EF21 paper): per worker, the better of the plain compressor b = C(s) and the
// Markov compressor m = g_i + C(s - g_i), s = grad f_i(x), C = Top-k.  The two Top-k selections are the
// library's ordinary ones; this file holds what is particular to Algorithm 3:
//   line 7  the distortions B = ||b - s||^2 = ||s||^2 - sum of the kept s_j^2 and
//           M = ||m - s||^2 = ||s - g_i||^2 - sum of the kept (s_j - g_ij)^2 (at a kept position m_j equals s_j
//           up to the rounding of one fp32 addition), differences and sums in fp64, in a fixed order;
//   line 8  g_i <- m if M <= B, else b: a sparse update, or a rewrite of the whole row;
//   line 10 g = (1/n) sum_i g_i is then recomputed from the rows (launch_mean_rows).
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
// exactly (in fp64), as the distortions of line 7 are defined on the stored vectors.
__global__ __launch_bounds__(kThreads) void plus_sqnorms_kernel(const float *__restrict__ s,
                                                                const float *__restrict__ g_i, int64_t d,
                                                                double2 *__restrict__ part) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.y, chunk = blockIdx.x;
    const int64_t lo = chunk * kNormChunk, hi = lo + kNormChunk < d ? lo + kNormChunk : d;
    const float *sr = s + row * d, *gr = g_i + row * d;
    double acc_s = 0.0, acc_v = 0.0;
    for (int64_t e = lo + threadIdx.x; e < hi; e += kThreads) {
        const double sv = (double)stream_load(sr + e), v = sv - (double)stream_load(gr + e);   // exact
        acc_s += sv * sv;
        acc_v += v * v;
    }
    acc_s = block_sum_f64(acc_s, lds);
    acc_v = block_sum_f64(acc_v, lds);
    if (threadIdx.x == 0) part[row * gridDim.x + chunk] = make_double2(acc_s, acc_v);
}

// One workgroup per worker: B, M, the choice of line 8, and the chosen message copied to (msg_idx, msg_val).
__global__ __launch_bounds__(kThreads) void plus_decide_kernel(const float *__restrict__ s,
                                                               const float *__restrict__ g_i, int64_t d,
                                                               const double2 *__restrict__ part, int64_t chunks,
                                                               const int32_t *__restrict__ idx_b,
                                                               const float *__restrict__ val_b,
                                                               const int32_t *__restrict__ idx_m,
                                                               const float *__restrict__ val_m, int64_t k,
                                                               int32_t *__restrict__ branch, double *__restrict__ BM,
                                                               int32_t *__restrict__ msg_idx,
                                                               float *__restrict__ msg_val) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.x;
    double ns = 0.0, nv = 0.0, kb = 0.0, km = 0.0;
    for (int64_t c = threadIdx.x; c < chunks; c += kThreads) {
        const double2 p = part[row * chunks + c];
        ns += p.x;
        nv += p.y;
    }
    for (int64_t j = threadIdx.x; j < k; j += kThreads) {
        // what the kept entries take away from the two norms: b_j = s_j exactly; m_j = s_j up to the rounding
        // of the fp32 update, so the exact (s_j - g_ij)^2 leaves the sum
        const double vb = (double)val_b[row * k + j];
        const int64_t e = idx_m[row * k + j];
        const double vm = (double)s[row * d + e] - (double)g_i[row * d + e];
        kb += vb * vb;
        km += vm * vm;
    }
    ns = block_sum_f64(ns, lds);
    nv = block_sum_f64(nv, lds);
    kb = block_sum_f64(kb, lds);
    km = block_sum_f64(km, lds);
    const double B = ns - kb, M = nv - km;
    const bool plain = M > B;                       // line 8: the Markov compressor unless it is strictly worse
    if (threadIdx.x == 0) {
        branch[row] = plain ? 1 : 0;
        BM[2 * row] = B;
        BM[2 * row + 1] = M;
    }
    const int32_t *ci = plain ? idx_b : idx_m;
    const float *cv = plain ? val_b : val_m;
    for (int64_t j = threadIdx.x; j < k; j += kThreads) {
        msg_idx[row * k + j] = ci[row * k + j];
        msg_val[row * k + j] = cv[row * k + j];
    }
}

// Rows whose worker chose the plain compressor are cleared (g_i <- b has k non-zeros at most).
__global__ __launch_bounds__(kThreads) void plus_clear_kernel(const int32_t *__restrict__ branch,
                                                              float *__restrict__ g_i, int64_t d) {
    const int64_t row = blockIdx.y;
    if (!branch[row]) return;
    const int64_t lo = (int64_t)blockIdx.x * kNormChunk, hi = lo + kNormChunk < d ? lo + kNormChunk : d;
    float *gr = g_i + row * d;
    for (int64_t e = lo + threadIdx.x; e < hi; e += kThreads) gr[e] = 0.f;
}

// The k entries of the chosen message: added to g_i (Markov branch, one fp32 addition each) or written
// into the cleared row (plain branch).
__global__ __launch_bounds__(kThreads) void plus_apply_kernel(const int32_t *__restrict__ branch,
                                                              const int32_t *__restrict__ msg_idx,
                                                              const float *__restrict__ msg_val, int64_t k,
                                                              float *__restrict__ g_i, int64_t d) {
    const int64_t row = blockIdx.y;
    const bool plain = branch[row] != 0;
    float *gr = g_i + row * d;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < k; j += stride) {
        const int32_t e = msg_idx[row * k + j];
        const float v = msg_val[row * k + j];
        gr[e] = plain ? v : gr[e] + v;
    }
}

int64_t chunks_of(int64_t d) { return (d + kNormChunk - 1) / kNormChunk; }

}  // namespace

size_t plus_scratch_bytes(int32_t n, int64_t d) { return sizeof(double2) * (size_t)n * (size_t)chunks_of(d); }

hipError_t launch_plus_choose(const float *s, float *g_i, int32_t n, int64_t d, int64_t k, const int32_t *idx_b,
                              const float *val_b, const int32_t *idx_m, const float *val_m, void *scratch,
                              int32_t *branch, double *BM, int32_t *msg_idx, float *msg_val, hipStream_t stream) {
    const int64_t chunks = chunks_of(d);
    double2 *part = (double2 *)scratch;
    hipLaunchKernelGGL(plus_sqnorms_kernel, dim3((unsigned)chunks, (unsigned)n), dim3(kThreads), 0, stream, s, g_i, d,
                       part);
    hipLaunchKernelGGL(plus_decide_kernel, dim3((unsigned)n), dim3(kThreads), 0, stream, s, g_i, d, part, chunks, idx_b, val_b,
                       idx_m, val_m, k, branch, BM, msg_idx, msg_val);
    hipLaunchKernelGGL(plus_clear_kernel, dim3((unsigned)chunks, (unsigned)n), dim3(kThreads), 0, stream, branch, g_i,
                       d);
    int64_t blocks = (k + kThreads - 1) / kThreads;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(plus_apply_kernel, dim3((unsigned)blocks, (unsigned)n), dim3(kThreads), 0, stream, branch,
                       msg_idx, msg_val, k, g_i, d);
    return hipGetLastError();
}

}  // namespace ef21
