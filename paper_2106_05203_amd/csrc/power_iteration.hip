// Power iteration for the smoothness constants of Section 3.4 (the L_i of the smoothness assumption and the L
// of f) that the stepsize of Theorem 1 is made of.  The products w = (1/m) A_i^T A_i v come from the gradient
// kernels (per-row loss z^2 / 2); this file holds the start vector and the step v <- w / |w| with the two
// numbers it yields, v^T w and |w| (both at most the largest eigenvalue for a unit v, |w| the closer one).
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ double block_sum_f64(double v, double *lds) {
    v = wave_sum_f64(v);
    __syncthreads();
    if (lane_id() == 0) lds[threadIdx.x / kWave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < kWaves; ++w) t += lds[w];
    return t;
}

// A fixed start vector of unit length with every entry positive and no two neighbours alike: entries in
// [0.5, 1.5) from an integer hash of the position, scaled by 1 / sqrt(d) (its length is then within [0.5, 1.5)).
__global__ __launch_bounds__(kThreads) void power_start_kernel(float *__restrict__ v, int64_t d) {
    const int64_t row = blockIdx.y;
    const float scale = rsqrtf((float)d);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < d; j += stride) {
        uint32_t h = (uint32_t)j * 2654435761u + 0x9e3779b9u * (uint32_t)(row + 1);
        h ^= h >> 15;
        h *= 2246822519u;
        h ^= h >> 13;
        v[row * d + j] = (0.5f + (float)(h >> 8) * (1.0f / 16777216.0f)) * scale;
    }
}

// One workgroup per row: stats[row] = (v^T w / v^T v, |w| / |v|), then v <- w / |w| (left alone if w = 0).
__global__ __launch_bounds__(kThreads) void power_step_kernel(const float *__restrict__ w, float *__restrict__ v,
                                                              int64_t d, double2 *__restrict__ stats) {
    __shared__ double lds[kWaves];
    const int64_t row = blockIdx.x;
    const float *wr = w + row * d;
    float *vr = v + row * d;
    double vw = 0.0, ww = 0.0, vv = 0.0;
    for (int64_t j = threadIdx.x; j < d; j += kThreads) {
        const double a = (double)vr[j], b = (double)wr[j];
        vw += a * b;
        ww += b * b;
        vv += a * a;
    }
    vw = block_sum_f64(vw, lds);
    ww = block_sum_f64(ww, lds);
    vv = block_sum_f64(vv, lds);
    const double nw = sqrt(ww), nv = sqrt(vv);
    if (threadIdx.x == 0) stats[row] = make_double2(vv > 0.0 ? vw / vv : 0.0, nv > 0.0 ? nw / nv : 0.0);
    if (nw > 0.0) {
        const double inv = 1.0 / nw;
        for (int64_t j = threadIdx.x; j < d; j += kThreads) vr[j] = (float)((double)wr[j] * inv);
    }
}

}  // namespace

hipError_t launch_power_start(float *v, int32_t rows, int64_t d, hipStream_t stream) {
    int64_t blocks = (d + kThreads - 1) / kThreads;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(power_start_kernel, dim3((unsigned)blocks, (unsigned)rows), dim3(kThreads), 0, stream, v, d);
    return hipGetLastError();
}

hipError_t launch_power_step(const float *w, float *v, int32_t rows, int64_t d, double *stats, hipStream_t stream) {
    hipLaunchKernelGGL(power_step_kernel, dim3((unsigned)rows), dim3(kThreads), 0, stream, w, v, d, (double2 *)stats);
    return hipGetLastError();
}

}  // namespace ef21
