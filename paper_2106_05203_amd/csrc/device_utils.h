// Wavefront-level helpers shared by the HIP kernels (gfx950: 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ef21 {

constexpr int kWave = 64;

// Magnitude key of Top-k: the fp32 bit pattern with the sign cleared.  For non-NaN values the
// unsigned order of keys is the order of |v|, +a and -a share a key, so do +0 and -0.
__device__ __forceinline__ uint32_t mag_key(float v) { return __float_as_uint(v) & 0x7fffffffu; }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// number of set bits of `mask` in lanes below the caller's
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint32_t popc64(uint64_t m) { return (uint32_t)__popcll(m); }

// Loads of streamed data (read once by the kernel, too large to stay in a cache): marked non-temporal
// so that the lines are not kept.  stream_load4 needs a 16-byte aligned address.
__device__ __forceinline__ float4 stream_load4(const float *p) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ float stream_load(const float *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ int32_t stream_load(const int32_t *p) { return __builtin_nontemporal_load(p); }

// Derivative in z of the per-row loss of a linear model, z = a^T x:
//   kLossLogistic       log(1 + exp(-y z))  (Section 5, eq. (9)):   -y / (1 + exp(y z))
//   kLossLeastSquares   (z - y)^2           (Section 5.2):          2 (z - y)
//   kLossHalfSquare     z^2 / 2 (no target; its "gradient" is (1/m) A^T A x, used by the power iteration): z
__device__ __forceinline__ float loss_derivative(float y, float z, int loss) {
    if (loss == 2 /* kLossHalfSquare */) return z;
    return loss == 1 /* kLossLeastSquares */ ? 2.0f * (z - y) : -y / (1.0f + expf(y * z));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Place of the calling lane's item in a list whose length is `*counter` (LDS): the lanes of a wavefront that
// have an item (`has`) take consecutive places with ONE atomic for the wavefront.  Every lane of the wavefront
// must call; the result means something only where `has`.
__device__ __forceinline__ uint32_t wave_append(bool has, uint32_t *counter) {
    const uint64_t m = __ballot(has);
    if (m == 0) return 0u;
    const int first = __ffsll((long long)m) - 1;
    uint32_t base = 0u;
    if (lane_id() == first) base = atomicAdd(counter, popc64(m));
    return __shfl(base, first, kWave) + lanes_below(m);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint32_t t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}

}  // namespace ef21
