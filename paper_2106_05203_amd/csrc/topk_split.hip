// Batched Top-k (Section 2.1 of the EF21 paper) for long rows: many workgroups per row.
//
// Same selection rule as the one-workgroup kernel (31-bit magnitude key, digits of 12 + 10 + 9
// bits, ties to the lower index, ascending output), organised so that the row itself is read
// twice and everything else touches only the few per cent of entries that can still be selected:
//
//   hist     full read   12-bit LDS histogram per workgroup, merged with atomics; the last
//                        workgroup of a row finds the digit d1 that holds the k-th magnitude
//   collect  full read   every entry whose first digit is >= d1 is a candidate; each wavefront
//                        owns a fixed segment of the row and appends its candidates, in position
//                        order, to its own slot of the workspace; second-digit histogram of the
//                        d1 bin on the side; last workgroup of a row finds d2
//   refine   candidates  third-digit histogram -> threshold key T and tie quota q
//   count    candidates  per slot: entries above T, entries equal to T; last workgroup of a row
//                        scans the slots into output offsets and tie ranks
//   emit     candidates  ordered write of the k kept entries (+ lines 6 and 8 of Algorithm 2)
//
// Slots have the capacity of their segment, so any input fits (all-equal rows included) and no
// fallback path exists.  "Last workgroup of a row" is decided with one atomic ticket per
// workgroup after a device-scope fence; nobody waits on anybody.  Histograms and tickets are
// left zeroed by the workgroup that consumes them, so the workspace needs zeroing only once.
#include "device_utils.h"
#include "kernels.h"

namespace ef21 {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kSegLen = 4096;                 // entries per wavefront segment = slot capacity
constexpr int kBits1 = 12, kBits2 = 10, kBits3 = 9;
constexpr int kBins1 = 1 << kBits1, kBins2 = 1 << kBits2, kBins3 = 1 << kBits3;

struct RowInfo {
    uint32_t d1, need1;   // first digit of the threshold; entries still needed from that bin
    uint32_t p22, need2;  // first two digits; entries still needed from that sub-bin
    uint32_t T, q;        // threshold key; number of entries equal to T to keep
    uint32_t pad0, pad1;
};

struct Ws {
    uint32_t *hist1, *hist2, *hist3;   // [n][bins]
    uint32_t *ticket;                  // [n][4]
    RowInfo *info;                     // [n]
    uint32_t *slot_cnt, *slot_gt, *slot_eq, *slot_off, *slot_eqb;   // [n][nseg]
    int32_t *cand_idx;                 // [n][nseg][kSegLen]
    float *cand_val;
    int64_t nseg;                      // segments (slots) per row
    int64_t nblk;                      // workgroups per row
};

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

size_t layout(int32_t n, int64_t d, char *base, Ws *w) {
    const int64_t nseg = (d + kSegLen - 1) / kSegLen;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += align256(bytes);
        return p;
    };
    char *h1 = take(sizeof(uint32_t) * (size_t)n * kBins1);
    char *h2 = take(sizeof(uint32_t) * (size_t)n * kBins2);
    char *h3 = take(sizeof(uint32_t) * (size_t)n * kBins3);
    char *tk = take(sizeof(uint32_t) * (size_t)n * 4);
    char *inf = take(sizeof(RowInfo) * (size_t)n);
    const size_t slots = sizeof(uint32_t) * (size_t)n * nseg;
    char *s0 = take(slots), *s1 = take(slots), *s2 = take(slots), *s3 = take(slots), *s4 = take(slots);
    char *ci = take(sizeof(int32_t) * (size_t)n * nseg * kSegLen);
    char *cv = take(sizeof(float) * (size_t)n * nseg * kSegLen);
    if (w) {
        w->hist1 = (uint32_t *)h1; w->hist2 = (uint32_t *)h2; w->hist3 = (uint32_t *)h3;
        w->ticket = (uint32_t *)tk; w->info = (RowInfo *)inf;
        w->slot_cnt = (uint32_t *)s0; w->slot_gt = (uint32_t *)s1; w->slot_eq = (uint32_t *)s2;
        w->slot_off = (uint32_t *)s3; w->slot_eqb = (uint32_t *)s4;
        w->cand_idx = (int32_t *)ci; w->cand_val = (float *)cv;
        w->nseg = nseg;
        w->nblk = (nseg + kWaves - 1) / kWaves;
    }
    return off;
}

// ---------------------------------------------------------------- workgroup-level helpers
// exclusive prefix sum over the workgroup's threads; total returned through *total
__device__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *lds_wave /*[kWaves]*/, uint32_t *total) {
    const uint32_t incl = wave_inclusive_scan(v);
    const int wave = threadIdx.x / kWave;
    __syncthreads();                       // lds_wave may still be in use by a previous scan
    if (lane_id() == kWave - 1) lds_wave[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = lds_wave[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// Takes a ticket for `row`; true in every thread of the workgroup that arrives last.
// All global writes of the workgroup made before the call are visible to that last workgroup.
__device__ bool last_block_of_row(uint32_t *ticket, uint32_t blocks, uint32_t *lds_flag) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = atomicAdd(ticket, 1u);
        *lds_flag = (t == blocks - 1) ? 1u : 0u;
        if (t == blocks - 1) *ticket = 0u;     // ready for the next call
    }
    __syncthreads();
    const bool last = *lds_flag != 0u;
    if (last) __threadfence();
    return last;
}

// Digit selection over a merged histogram in global memory, by the last workgroup of a row:
// largest bin b with count(bins > b) < need <= count(bins >= b).  Zeroes the histogram.
// Results in lds_out[0] = b, lds_out[1] = need - count(bins > b).
template <int NBINS>
__device__ void select_digit(uint32_t *hist, uint32_t need, uint32_t *lds_wave, uint32_t *lds_out) {
    constexpr int PER = NBINS / kThreads;      // bins per thread, walked from the top
    static_assert(PER >= 1 && PER * kThreads == NBINS, "histogram size must be a multiple of the workgroup");
    uint32_t h[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int bin = NBINS - 1 - ((int)threadIdx.x * PER + j);
        h[j] = __hip_atomic_load(hist + bin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        hist[bin] = 0u;
        mine += h[j];
    }
    uint32_t total;
    const uint32_t above = block_exclusive_scan(mine, lds_wave, &total);
    if (above < need && need <= above + mine) {
        uint32_t c = above;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (need > c && need <= c + h[j]) {
                lds_out[0] = (uint32_t)(NBINS - 1 - ((int)threadIdx.x * PER + j));
                lds_out[1] = need - c;
            }
            c += h[j];
        }
    }
    __syncthreads();
}

// Adds a workgroup's LDS histogram into the row's global one (non-empty bins only).
template <int NBINS>
__device__ void flush_hist(const uint32_t *lds_hist, uint32_t *global_hist) {
    for (int b = threadIdx.x; b < NBINS; b += kThreads) {
        const uint32_t c = lds_hist[b];
        if (c) atomicAdd(global_hist + b, c);
    }
}

// ---------------------------------------------------------------- segment reader
// A wavefront walks its segment in steps of 64*VEC entries.  VEC = 4 needs 16-byte aligned rows.
// Entry order inside a step: lane-major, then the VEC entries of the lane.
template <int VEC, bool DIFF>
struct Step {
    float v[VEC];
    __device__ __forceinline__ void load(const float *a, const float *b, int64_t e0, int64_t end) {
        if constexpr (VEC == 4) {
            if (e0 + 3 < end) {
                const float4 t = *reinterpret_cast<const float4 *>(a + e0);
                v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                if constexpr (DIFF) {
                    const float4 s = *reinterpret_cast<const float4 *>(b + e0);
                    v[0] -= s.x; v[1] -= s.y; v[2] -= s.z; v[3] -= s.w;
                }
                return;
            }
        }
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            v[t] = 0.f;
            if (e0 + t < end) {
                v[t] = a[e0 + t];
                if constexpr (DIFF) v[t] -= b[e0 + t];
            }
        }
    }
};

// ---------------------------------------------------------------- kernel 1: first-digit histogram
template <int VEC, bool DIFF>
__global__ __launch_bounds__(kThreads) void split_hist_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t hist[kBins1];
    __shared__ uint32_t lds_wave[kWaves], lds_out[2], lds_flag;
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    for (int i = threadIdx.x; i < kBins1; i += kThreads) hist[i] = 0u;
    __syncthreads();

    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t lo = seg * kSegLen;
    const int64_t hi = lo + kSegLen < d ? lo + kSegLen : d;
    constexpr int kStep = kWave * VEC, kUnroll = 4;
    for (int64_t base = lo; base < hi; base += kStep * kUnroll) {
        Step<VEC, DIFF> st[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) st[u].load(a, b, base + u * kStep + lane * VEC, hi);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int t = 0; t < VEC; ++t)
                if (base + u * kStep + lane * VEC + t < hi)
                    atomicAdd(&hist[mag_key(st[u].v[t]) >> (kBits2 + kBits3)], 1u);
    }
    __syncthreads();
    flush_hist<kBins1>(hist, w.hist1 + row * kBins1);

    if (last_block_of_row(w.ticket + row * 4 + 0, (uint32_t)w.nblk, &lds_flag)) {
        select_digit<kBins1>(w.hist1 + row * kBins1, (uint32_t)p.k, lds_wave, lds_out);
        if (threadIdx.x == 0) {
            w.info[row].d1 = lds_out[0];
            w.info[row].need1 = lds_out[1];
        }
    }
}

// ---------------------------------------------------------------- kernel 2: collect candidates
template <int VEC, bool DIFF>
__global__ __launch_bounds__(kThreads) void split_collect_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t hist[kBins2];
    __shared__ uint32_t lds_wave[kWaves], lds_out[2], lds_flag;
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    for (int i = threadIdx.x; i < kBins2; i += kThreads) hist[i] = 0u;
    __syncthreads();
    const uint32_t d1 = w.info[row].d1;
    const uint32_t key_lo = d1 << (kBits2 + kBits3);          // smallest candidate key

    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kWaves + wave;
    const int64_t lo = seg * kSegLen;
    const int64_t hi = lo + kSegLen < d ? lo + kSegLen : d;
    if (seg < w.nseg) {
        int32_t *slot_idx = w.cand_idx + (row * w.nseg + seg) * kSegLen;
        float *slot_val = w.cand_val + (row * w.nseg + seg) * kSegLen;
        uint32_t cnt = 0;
        constexpr int kStep = kWave * VEC, kUnroll = 4;
        for (int64_t base = lo; base < hi; base += kStep * kUnroll) {
            Step<VEC, DIFF> st[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) st[u].load(a, b, base + u * kStep + lane * VEC, hi);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t e0 = base + u * kStep + lane * VEC;
                bool c[VEC];
                uint32_t below = 0, all = 0;
#pragma unroll
                for (int t = 0; t < VEC; ++t) {
                    const uint32_t key = mag_key(st[u].v[t]);
                    c[t] = (e0 + t < hi) && key >= key_lo;
                    const uint64_t m = __ballot(c[t]);
                    below += lanes_below(m);
                    all += popc64(m);
                }
                if (all) {
                    uint32_t pos = cnt + below;
#pragma unroll
                    for (int t = 0; t < VEC; ++t) {
                        if (c[t]) {
                            slot_idx[pos] = (int32_t)(e0 + t);
                            slot_val[pos] = st[u].v[t];
                            const uint32_t key = mag_key(st[u].v[t]);
                            if ((key >> (kBits2 + kBits3)) == d1) atomicAdd(&hist[(key >> kBits3) & (kBins2 - 1)], 1u);
                            ++pos;
                        }
                    }
                    cnt += all;
                }
            }
        }
        if (lane == 0) w.slot_cnt[row * w.nseg + seg] = cnt;
    }
    __syncthreads();
    flush_hist<kBins2>(hist, w.hist2 + row * kBins2);

    if (last_block_of_row(w.ticket + row * 4 + 1, (uint32_t)w.nblk, &lds_flag)) {
        select_digit<kBins2>(w.hist2 + row * kBins2, w.info[row].need1, lds_wave, lds_out);
        if (threadIdx.x == 0) {
            w.info[row].p22 = (d1 << kBits2) | lds_out[0];
            w.info[row].need2 = lds_out[1];
        }
    }
}

// ---------------------------------------------------------------- kernel 3: third digit -> T, q
__global__ __launch_bounds__(kThreads) void split_refine_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t hist[kBins3];
    __shared__ uint32_t lds_wave[kWaves], lds_out[2], lds_flag;
    const int64_t row = blockIdx.y;
    for (int i = threadIdx.x; i < kBins3; i += kThreads) hist[i] = 0u;
    __syncthreads();
    const uint32_t p22 = w.info[row].p22;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kWaves + wave;
    if (seg < w.nseg) {
        const uint32_t cnt = w.slot_cnt[row * w.nseg + seg];
        const float *slot_val = w.cand_val + (row * w.nseg + seg) * kSegLen;
        for (uint32_t j = lane; j < cnt; j += kWave) {
            const uint32_t key = mag_key(slot_val[j]);
            if ((key >> kBits3) == p22) atomicAdd(&hist[key & (kBins3 - 1)], 1u);
        }
    }
    __syncthreads();
    flush_hist<kBins3>(hist, w.hist3 + row * kBins3);

    if (last_block_of_row(w.ticket + row * 4 + 2, (uint32_t)w.nblk, &lds_flag)) {
        select_digit<kBins3>(w.hist3 + row * kBins3, w.info[row].need2, lds_wave, lds_out);
        if (threadIdx.x == 0) {
            w.info[row].T = (p22 << kBits3) | lds_out[0];
            w.info[row].q = lds_out[1];
        }
    }
    (void)p;
}

// ---------------------------------------------------------------- kernel 4: per-slot counts, offsets
__global__ __launch_bounds__(kThreads) void split_count_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t lds_wave[kWaves], lds_flag;
    const int64_t row = blockIdx.y;
    const uint32_t T = w.info[row].T;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kWaves + wave;
    if (seg < w.nseg) {
        const uint32_t cnt = w.slot_cnt[row * w.nseg + seg];
        const float *slot_val = w.cand_val + (row * w.nseg + seg) * kSegLen;
        uint32_t n_gt = 0, n_eq = 0;
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const uint32_t j = j0 + lane;
            const uint32_t key = j < cnt ? mag_key(slot_val[j]) : 0u;
            n_gt += popc64(__ballot(j < cnt && key > T));
            n_eq += popc64(__ballot(j < cnt && key == T));
        }
        if (lane == 0) {
            w.slot_gt[row * w.nseg + seg] = n_gt;
            w.slot_eq[row * w.nseg + seg] = n_eq;
        }
    }
    if (last_block_of_row(w.ticket + row * 4 + 3, (uint32_t)w.nblk, &lds_flag)) {
        // exclusive scans over the row's slots, in slot order
        const uint32_t q = w.info[row].q;
        const int64_t nseg = w.nseg;
        const int64_t per = (nseg + kThreads - 1) / kThreads;
        const int64_t s0 = (int64_t)threadIdx.x * per;
        const int64_t s1 = s0 + per < nseg ? s0 + per : nseg;
        uint32_t my_gt = 0, my_eq = 0;
        for (int64_t s = s0; s < s1; ++s) {
            my_gt += __hip_atomic_load(w.slot_gt + row * nseg + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            my_eq += __hip_atomic_load(w.slot_eq + row * nseg + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        uint32_t tot;
        uint32_t gt_run = block_exclusive_scan(my_gt, lds_wave, &tot);
        uint32_t eq_run = block_exclusive_scan(my_eq, lds_wave, &tot);
        for (int64_t s = s0; s < s1; ++s) {
            const uint32_t g = __hip_atomic_load(w.slot_gt + row * nseg + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint32_t e = __hip_atomic_load(w.slot_eq + row * nseg + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            w.slot_off[row * nseg + s] = gt_run + (eq_run < q ? eq_run : q);   // kept entries before slot
            w.slot_eqb[row * nseg + s] = eq_run;                               // ties before slot
            gt_run += g;
            eq_run += e;
        }
    }
    (void)p;
}

// ---------------------------------------------------------------- kernel 5: ordered emission
template <bool UPDATE>
__global__ __launch_bounds__(kThreads) void split_emit_kernel(TopkArgs p, Ws w) {
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t seg = (int64_t)blockIdx.x * kWaves + wave;
    if (seg >= w.nseg) return;
    const uint32_t T = w.info[row].T, q = w.info[row].q;
    const uint32_t cnt = w.slot_cnt[row * w.nseg + seg];
    uint32_t out_run = w.slot_off[row * w.nseg + seg];
    uint32_t eq_run = w.slot_eqb[row * w.nseg + seg];
    const int32_t *slot_idx = w.cand_idx + (row * w.nseg + seg) * kSegLen;
    const float *slot_val = w.cand_val + (row * w.nseg + seg) * kSegLen;
    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
        const uint32_t j = j0 + lane;
        const bool in = j < cnt;
        const float v = in ? slot_val[j] : 0.f;
        const uint32_t key = mag_key(v);
        const bool gt = in && key > T, eq = in && key == T;
        const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
        const uint32_t eq_below = eq_run + lanes_below(m_eq);
        const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
        if (gt || (eq && eq_below < q)) {
            const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
            const int32_t e = slot_idx[j];
            out_idx[pos] = e;
            out_val[pos] = v;
            if (UPDATE) {
                float *g_i = p.g_i + row * p.d;
                g_i[e] = g_i[e] + v;                   // Algorithm 2, line 6 (g_i still holds its old value)
                atomicAdd(p.g + e, v * p.inv_n);       // Algorithm 2, line 8
            }
        }
        const uint32_t eq_next = eq_run + popc64(m_eq);
        out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_run < q ? eq_run : q));
        eq_run = eq_next;
    }
}

__global__ __launch_bounds__(kThreads) void zero_words_kernel(uint32_t *p, size_t words) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

template <int VEC, bool DIFF>
void launch_front(const TopkArgs &p, const Ws &w, dim3 grid, hipStream_t stream, const Marker &mk) {
    hipLaunchKernelGGL((split_hist_kernel<VEC, DIFF>), grid, dim3(kThreads), 0, stream, p, w);
    mk(K_TOPK_HIST);
    hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF>), grid, dim3(kThreads), 0, stream, p, w);
    mk(K_TOPK_COLLECT);
}

}  // namespace

size_t topk_split_workspace_bytes(int32_t n, int64_t d, int64_t) { return layout(n, d, nullptr, nullptr); }

hipError_t launch_topk_split_reset(void *workspace, int32_t n, int64_t d, hipStream_t stream) {
    Ws w;
    layout(n, d, (char *)workspace, &w);
    // histograms and tickets are the leading, contiguous part of the layout
    const size_t words = ((char *)w.info - (char *)workspace) / sizeof(uint32_t);
    size_t blocks = (words + kThreads - 1) / kThreads;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, (uint32_t *)workspace,
                       words);
    return hipGetLastError();
}

hipError_t launch_topk_split(const TopkArgs &p, void *workspace, hipStream_t stream, const Marker &mk) {
    Ws w;
    layout(p.n, p.d, (char *)workspace, &w);
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    if (upd && !diff) return hipErrorInvalidValue;
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0) && (!diff || (uintptr_t)p.b % 16 == 0);
    const dim3 grid((unsigned)w.nblk, (unsigned)p.n);
    if (vec4 && diff) launch_front<4, true>(p, w, grid, stream, mk);
    else if (vec4) launch_front<4, false>(p, w, grid, stream, mk);
    else if (diff) launch_front<1, true>(p, w, grid, stream, mk);
    else launch_front<1, false>(p, w, grid, stream, mk);
    hipLaunchKernelGGL(split_refine_kernel, grid, dim3(kThreads), 0, stream, p, w);
    mk(K_TOPK_REFINE);
    hipLaunchKernelGGL(split_count_kernel, grid, dim3(kThreads), 0, stream, p, w);
    mk(K_TOPK_COUNT);
    if (upd) hipLaunchKernelGGL(split_emit_kernel<true>, grid, dim3(kThreads), 0, stream, p, w);
    else hipLaunchKernelGGL(split_emit_kernel<false>, grid, dim3(kThreads), 0, stream, p, w);
    mk(K_TOPK_EMIT);
    return hipGetLastError();
}

}  // namespace ef21
