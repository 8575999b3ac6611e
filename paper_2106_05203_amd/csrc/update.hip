// Dense vector kernels of Algorithm 2: the model step (line 3) and the mean of the workers'
// estimators (input line, g^0 = (1/n) sum_i g_i^0).
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;

// x_j <- x_j - gamma g_j as one fused multiply-add per coordinate (a single rounding).
__global__ __launch_bounds__(kThreads) void model_step_kernel(float *__restrict__ x, const float *__restrict__ g,
                                                              int64_t d, float neg_gamma) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < d; j += stride)
        x[j] = fmaf(neg_gamma, g[j], x[j]);
}

// Same, four coordinates per lane; needs d % 4 == 0 and 16-byte aligned pointers.
__global__ __launch_bounds__(kThreads) void model_step_vec4_kernel(float4 *__restrict__ x,
                                                                   const float4 *__restrict__ g, int64_t d4,
                                                                   float neg_gamma) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < d4; j += stride) {
        float4 xv = x[j];
        const float4 gv = g[j];
        xv.x = fmaf(neg_gamma, gv.x, xv.x);
        xv.y = fmaf(neg_gamma, gv.y, xv.y);
        xv.z = fmaf(neg_gamma, gv.z, xv.z);
        xv.w = fmaf(neg_gamma, gv.w, xv.w);
        x[j] = xv;
    }
}

__global__ __launch_bounds__(kThreads) void mean_rows_kernel(const float *__restrict__ g_i, float *__restrict__ g,
                                                             int32_t n, int64_t d) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < d; j += stride) {
        double s = 0.0;
        for (int32_t i = 0; i < n; ++i) s += (double)g_i[(int64_t)i * d + j];
        g[j] = (float)(s / (double)n);
    }
}

unsigned grid_for(int64_t items, int64_t cap) {
    int64_t blocks = (items + kThreads - 1) / kThreads;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

}  // namespace

hipError_t launch_model_step(float *x, const float *g, int64_t d, float gamma, hipStream_t stream) {
    const bool vec = (d % 4 == 0) && (((uintptr_t)x | (uintptr_t)g) % 16 == 0);
    if (vec) {
        hipLaunchKernelGGL(model_step_vec4_kernel, dim3(grid_for(d / 4, 8192)), dim3(kThreads), 0, stream,
                           (float4 *)x, (const float4 *)g, d / 4, -gamma);
    } else {
        hipLaunchKernelGGL(model_step_kernel, dim3(grid_for(d, 8192)), dim3(kThreads), 0, stream, x, g, d,
                           -gamma);
    }
    return hipGetLastError();
}

hipError_t launch_mean_rows(const float *g_i, float *g, int32_t n, int64_t d, hipStream_t stream) {
    hipLaunchKernelGGL(mean_rows_kernel, dim3(grid_for(d, 8192)), dim3(kThreads), 0, stream, g_i, g, n, d);
    return hipGetLastError();
}

}  // namespace ef21
