// Batched Top-k (Section 2.1 of the EF21 paper), one workgroup per row.
//
// The k largest magnitudes of a row are found by a radix select on the 31-bit magnitude key
// (fp32 bits with the sign cleared): three histogram passes (12 + 10 + 9 bits, LDS histograms)
// fix the key T of the k-th largest magnitude and the number q of entries equal to T that are
// still needed; an ordered emission then writes every entry with key > T and the first q
// entries with key == T, in ascending position order (ties go to the lower index).
// With `g_i != nullptr` the emission also applies line 6 of Algorithm 2.
#include "topk_row_impl.h"

namespace ef21 {
namespace {

template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kRowThreads) void topk_row_kernel(TopkArgs p) {
    __shared__ RowShared s;
    row_topk<DIFF, UPDATE>(s, p, blockIdx.x);
}

template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kRowThreads) void topk_row_cached_kernel(TopkArgs p) {
    __shared__ RowShared s;
    __shared__ float cache[kRowCache];
    row_topk_cached<DIFF, UPDATE>(s, cache, p, blockIdx.x);
}

template <bool UPDATE>
__global__ __launch_bounds__(kRowThreads) void topk_row_parts_kernel(TopkArgs p) {
    __shared__ RowShared s;
    __shared__ float cache[kRowCache];
    row_topk_parts<UPDATE>(s, cache, p, blockIdx.x);
}

}  // namespace

hipError_t launch_topk_row(const TopkArgs &p, hipStream_t stream) {
    const dim3 grid((unsigned)p.n), block(kRowThreads);
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    if (upd && !diff) return hipErrorInvalidValue;   // line 6 needs the subtracted g_i
    if (p.parts.part) {
        if (!diff || p.d > kRowCache) return hipErrorInvalidValue;
        if (upd) hipLaunchKernelGGL((topk_row_parts_kernel<true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((topk_row_parts_kernel<false>), grid, block, 0, stream, p);
        return hipGetLastError();
    }
    if (p.d <= kRowCache) {
        if (upd) hipLaunchKernelGGL((topk_row_cached_kernel<true, true>), grid, block, 0, stream, p);
        else if (diff) hipLaunchKernelGGL((topk_row_cached_kernel<true, false>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((topk_row_cached_kernel<false, false>), grid, block, 0, stream, p);
    } else {
        if (upd) hipLaunchKernelGGL((topk_row_kernel<true, true>), grid, block, 0, stream, p);
        else if (diff) hipLaunchKernelGGL((topk_row_kernel<true, false>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((topk_row_kernel<false, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace ef21
