// EF, the original error feedback (Algorithm 4 of the EF21 paper), kept beside EF21 as the method it is
// compared with.  One round at the current x, with the errors e_i in the place of EF21's g_i:
//   p_i = e_i + gamma grad f_i(x)   written over e_i (one fused multiply-add per entry; every entry changes,
//                                   unlike EF21's state, which changes in k places);
//   w_i = C(p_i)                    the library's Top-k on the rows of e;
//   e_i = p_i - w_i                 zero at the kept positions;
//   x   = x - (1/n) sum_i w_i       the aggregation pass of Algorithm 2's line 8 on a zeroed vector, step 1.
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void ef_accumulate_vec4_kernel(const float *__restrict__ s,
                                                                      float4 *__restrict__ e, int64_t n4,
                                                                      float gamma) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
        const float4 sv = stream_load4(s + 4 * i);
        float4 ev = e[i];
        ev.x = fmaf(gamma, sv.x, ev.x);
        ev.y = fmaf(gamma, sv.y, ev.y);
        ev.z = fmaf(gamma, sv.z, ev.z);
        ev.w = fmaf(gamma, sv.w, ev.w);
        e[i] = ev;
    }
}

__global__ __launch_bounds__(kThreads) void ef_accumulate_kernel(const float *__restrict__ s, float *__restrict__ e,
                                                                 int64_t total, float gamma) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride)
        e[i] = fmaf(gamma, s[i], e[i]);
}

__global__ __launch_bounds__(kThreads) void ef_clear_kept_kernel(const int32_t *__restrict__ idx, int64_t k,
                                                                 float *__restrict__ e, int64_t d) {
    const int64_t row = blockIdx.y;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < k; j += stride)
        e[row * d + idx[row * k + j]] = 0.f;
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float *__restrict__ v, int64_t d) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < d; i += stride) v[i] = 0.f;
}

unsigned blocks_for(int64_t items, int64_t cap) {
    int64_t b = (items + kThreads - 1) / kThreads;
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (unsigned)b;
}

}  // namespace

hipError_t launch_ef_accumulate(const float *s, float *e, int32_t n, int64_t d, float gamma, hipStream_t stream) {
    const int64_t total = (int64_t)n * d;
    if (total % 4 == 0 && (((uintptr_t)s | (uintptr_t)e) % 16 == 0))
        hipLaunchKernelGGL(ef_accumulate_vec4_kernel, dim3(blocks_for(total / 4, 8192)), dim3(kThreads), 0, stream, s,
                           (float4 *)e, total / 4, gamma);
    else
        hipLaunchKernelGGL(ef_accumulate_kernel, dim3(blocks_for(total, 8192)), dim3(kThreads), 0, stream, s, e, total,
                           gamma);
    return hipGetLastError();
}

hipError_t launch_ef_clear_kept(const int32_t *idx, int32_t n, int64_t k, float *e, int64_t d, hipStream_t stream) {
    hipLaunchKernelGGL(ef_clear_kept_kernel, dim3(blocks_for(k, 256), (unsigned)n), dim3(kThreads), 0, stream, idx, k, e,
                       d);
    return hipGetLastError();
}

hipError_t launch_fill_zero(float *v, int64_t d, hipStream_t stream) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(d, 4096)), dim3(kThreads), 0, stream, v, d);
    return hipGetLastError();
}

}  // namespace ef21
