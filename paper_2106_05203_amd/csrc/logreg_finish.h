// Last step of the dense gradient of eq. (9): one entry of grad f_i from the per-row-block partial sums
// of (sum_l r_l a_l).  Shared by the kernel that writes the gradient out and by the Top-k kernel that
// consumes it directly, so that both see the same bits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ef21 {

// part_w: the worker's partial sums [chunks][d]; c: the column.  The row blocks are added in fp64 in four
// interleaved chains (block b into chain b mod 4, ascending), the chains in order; then
// sum / m + 2 lambda x_c / (1 + x_c^2)^2, rounded once to fp32.
__device__ __forceinline__ float dense_grad_entry(const float *__restrict__ part_w, int64_t chunks, int64_t d,
                                                  int64_t c, float x_c, int64_t m, float lambda) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int64_t b = 0;
    for (; b + 8 <= chunks; b += 8) {          // eight loads in flight
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = part_w[(b + u) * d + c];
        s0 += (double)p[0];
        s1 += (double)p[1];
        s2 += (double)p[2];
        s3 += (double)p[3];
        s0 += (double)p[4];
        s1 += (double)p[5];
        s2 += (double)p[6];
        s3 += (double)p[7];
    }
    {                                           // up to seven blocks left; b is a multiple of 4
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = b + u < chunks ? part_w[(b + u) * d + c] : 0.f;
        if (b + 0 < chunks) s0 += (double)p[0];
        if (b + 1 < chunks) s1 += (double)p[1];
        if (b + 2 < chunks) s2 += (double)p[2];
        if (b + 3 < chunks) s3 += (double)p[3];
        if (b + 4 < chunks) s0 += (double)p[4];
        if (b + 5 < chunks) s1 += (double)p[5];
        if (b + 6 < chunks) s2 += (double)p[6];
    }
    double t = s0;
    t += s1;
    t += s2;
    t += s3;
    const double xj = (double)x_c, q = 1.0 + xj * xj;
    return (float)(t / (double)m + 2.0 * (double)lambda * xj / (q * q));
}

}  // namespace ef21
