// Batched Top-k (Section 2.1 of the EF21 paper) for rows of 16 384 to 61 440 entries and k <= 1024: one
// 1024-thread workgroup per row that reads the row from memory ONCE.
//
// One compute unit executes 64 lanes per clock, so every pass over a row of 50 000 entries costs a third of a
// microsecond per instruction and entry, and LDS atomics on a few hot addresses cost far more: after the one
// pass that streams the row, all work is done on a short list of candidates.
//
//   1  The row is streamed once; of every entry the 16 leading bits of its 31-bit magnitude key go to LDS
//      (2 bytes per entry), and every thread keeps the two largest it has seen.
//   2  The k-th largest of those 2048 values is one of k distinct entries, so the k-th largest entry of the row
//      is no smaller: its 16-bit prefix bounds the threshold from below.
//   3  The entries from that prefix upwards (about one per cent of the row) are gathered from LDS into a list
//      (16-bit prefix, position): first the 16-byte words that hold one are listed (one packed maximum per
//      word), then the lanes take one listed word each.
//   4  A histogram of the list gives the bin of the k-th largest magnitude, narrowed by the four further bits
//      if it is crowded; the list's entries in that bin are read again from memory with all their bits and
//      ranked against one another (larger key first, lower position first), which decides each of them.
//   5  The kept entries (those above the bin, and the first of the bin) set their bits in a bitmap of the row;
//      a prefix sum over the bitmap gives each its place in the ascending output; their values are read from
//      memory a second time.
// A list that overflows (rows with very many equal magnitudes) or a bin that stays crowded falls back to the
// general row kernel.  Rows given as a difference of two arrays (line 5 of Algorithm 2 inside ef21_step) do not come
// here: read cold from two arrays, one compute unit per row is slower than the many-workgroup path.
#include "topk_row_impl.h"

namespace ef21 {
namespace {

constexpr int kCandMax = kRowThreads;           // entries ranked directly
static_assert(3 * kCandMax + kRowThreads <= (1 << kBits1),
              "the candidates (8 bytes each), their ranks and the kept positions reuse the histogram's memory");
constexpr int kKeyShift = 15;                  // key >> 15: the 16 leading bits of the 31
constexpr int kSubBits = 4;                    // of which the last four are not in the 12-bit histogram
static_assert(31 - kKeyShift == kBits1 + kSubBits, "16 = 12 + 4");

struct Shared16 {
    RowShared s;                               // hist is reused for the listed words, the candidates, the result
    uint32_t sub[1 << kSubBits];
    uint32_t n_words;
};
static_assert(kRow16Max / 8 <= 65536 && sizeof(uint16_t) * 4096 <= sizeof(uint32_t) * (1 << kBits1), "the listed words fit the histogram's memory");

// The eight 16-bit entries of one 16-byte LDS word group.
__device__ __forceinline__ void unpack8(const uint4 &w, uint32_t (&k16)[8]) {
    k16[0] = w.x & 0xffffu;
    k16[1] = w.x >> 16;
    k16[2] = w.y & 0xffffu;
    k16[3] = w.y >> 16;
    k16[4] = w.z & 0xffffu;
    k16[5] = w.z >> 16;
    k16[6] = w.w & 0xffffu;
    k16[7] = w.w >> 16;
}

// The largest of the eight (packed 16-bit maxima: one instruction per pair of entries).  One compute unit
// executes 64 lanes per clock, so a pass over a row of 50 000 entries costs a third of a microsecond per
// instruction and entry: the scans below look at whole words first and at single entries only where it matters.
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t max8(const uint4 &w) {
    const us2 m = __builtin_elementwise_max(
        __builtin_elementwise_max(__builtin_bit_cast(us2, w.x), __builtin_bit_cast(us2, w.y)),
        __builtin_elementwise_max(__builtin_bit_cast(us2, w.z), __builtin_bit_cast(us2, w.w)));
    return m.x > m.y ? (uint32_t)m.x : (uint32_t)m.y;
}

constexpr int kChunks = (int)((kRow16Max / 8 + kRowThreads - 1) / kRowThreads);   // 16-byte LDS words per thread: 8
constexpr int kListMax = 4096;                 // gathered entries (step 3) ...
constexpr int kWordMax = 4096;                 // ... and 16-byte words that hold one

template <bool VEC4>
__global__ __launch_bounds__(kRowThreads) void topk_row16_kernel(TopkArgs p) {
    __shared__ Shared16 sh;
    __shared__ uint32_t list[kListMax];        // prefix << 16 | position
    uint16_t *words = reinterpret_cast<uint16_t *>(sh.s.hist);      // [kWordMax] numbers of 16-byte words, step 3 only
    extern __shared__ __attribute__((aligned(16))) uint16_t keys16[];       // [d rounded up to 8]
    RowShared &s = sh.s;
    const int64_t row = blockIdx.x, d = p.d;
    const int tid = threadIdx.x, lane = lane_id();
    const uint32_t k = (uint32_t)p.k;          // <= kRowThreads
    const float *a = p.a + row * d;

    // ---- the one pass over the row: 16-bit key prefixes to LDS; every thread keeps the largest it has seen
    for (int i = tid; i < (1 << kBits1); i += kRowThreads) s.hist[i] = 0u;
    if (tid < (1 << kSubBits)) sh.sub[tid] = 0u;
    uint32_t my_max = 0u, my_2nd = 0u;         // the two largest prefixes this thread has seen
    auto seen = [&](uint32_t k16) {
        const uint32_t lo = k16 < my_max ? k16 : my_max;
        my_max = k16 > my_max ? k16 : my_max;
        my_2nd = lo > my_2nd ? lo : my_2nd;
    };
    if constexpr (VEC4) {
        constexpr int kUnroll = 8;             // eight float4 loads per array in flight per thread
        constexpr int64_t kStep = (int64_t)kRowThreads * 4;
        int64_t e = (int64_t)tid * 4;
        for (; e + (kUnroll - 1) * kStep + 4 <= d; e += kUnroll * kStep) {
            float4 va[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) va[u] = stream_load4(a + e + u * kStep);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const float v[4] = {va[u].x, va[u].y, va[u].z, va[u].w};
                uint32_t k16[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    k16[t] = mag_key(v[t]) >> kKeyShift;
                    seen(k16[t]);
                }
                *reinterpret_cast<uint2 *>(keys16 + e + u * kStep) =
                    make_uint2(k16[0] | (k16[1] << 16), k16[2] | (k16[3] << 16));
            }
        }
        for (; e < d; e += kStep) {            // d % 4 == 0: whole float4s
            const float4 va = stream_load4(a + e);
            const float v[4] = {va.x, va.y, va.z, va.w};
            uint32_t k16[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                k16[t] = mag_key(v[t]) >> kKeyShift;
                seen(k16[t]);
            }
            *reinterpret_cast<uint2 *>(keys16 + e) = make_uint2(k16[0] | (k16[1] << 16), k16[2] | (k16[3] << 16));
        }
    } else {
        constexpr int kUnroll = 8;
        int64_t e = tid;
        for (; e + (int64_t)(kUnroll - 1) * kRowThreads < d; e += (int64_t)kUnroll * kRowThreads) {
            float v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) v[u] = a[e + (int64_t)u * kRowThreads];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint32_t k16 = mag_key(v[u]) >> kKeyShift;
                seen(k16);
                keys16[e + (int64_t)u * kRowThreads] = (uint16_t)k16;
            }
        }
        for (; e < d; e += kRowThreads) {
            const uint32_t k16 = mag_key(a[e]) >> kKeyShift;
            seen(k16);
            keys16[e] = (uint16_t)k16;
        }
    }
    // entries past d in the last 16-byte word: zero, and never counted (every scan below checks the position)
    if (tid < 8 && d + tid < ((d + 7) & ~(int64_t)7)) keys16[d + tid] = 0;
    __syncthreads();

    // ---- 2: a 16-bit prefix that cannot lie above the k-th largest: the k-th largest of the 2048 values "two
    // largest of a thread" (d >= 2048: 2048 distinct entries), by its bin and then by its last four bits
    atomicAdd(&s.hist[my_max >> kSubBits], 1u);
    atomicAdd(&s.hist[my_2nd >> kSubBits], 1u);
    if (tid == 0) {
        s.ncand = 0u;
        sh.n_words = 0u;
    }
    __syncthreads();
    select_bin(s, 1 << kBits1, k);
    uint32_t low16 = s.bin << kSubBits;
    {
        const uint32_t lb = s.bin, nb = s.need;              // nb of the values in bin lb are among the k largest
        __syncthreads();
        // counts of the sixteen sub-bins from ballots (an atomic per thread on sixteen addresses would queue up)
        const bool in1 = (my_max >> kSubBits) == lb, in2 = (my_2nd >> kSubBits) == lb;
        for (int sb = 0; sb < (1 << kSubBits); ++sb) {
            const uint32_t cnt = popc64(__ballot(in1 && (my_max & 15u) == (uint32_t)sb)) +
                                 popc64(__ballot(in2 && (my_2nd & 15u) == (uint32_t)sb));
            if (lane == 0 && cnt) atomicAdd(&sh.sub[sb], cnt);
        }
        __syncthreads();
        uint32_t above = 0u;
        for (int sb = (1 << kSubBits) - 1; sb >= 0; --sb) {  // every thread walks the sixteen counts
            const uint32_t h = sh.sub[sb];
            if (nb <= above + h) {
                low16 |= (uint32_t)sb;
                break;
            }
            above += h;
        }
        __syncthreads();
        if (tid < (1 << kSubBits)) sh.sub[tid] = 0u;         // used again in step 4
    }
    __syncthreads();                                         // the maxima's histogram is done with

    // ---- 3: the entries of at least low16, gathered.  First the 16-byte words that hold such an entry (one packed
    // maximum per word) are listed, then the lanes take one listed word each and append its entries: taking the
    // words apart where they lie would keep every lane busy for the sake of one in seven.
    const int64_t d8 = (d + 7) / 8;
    const uint4 *keys8 = reinterpret_cast<const uint4 *>(keys16);
    {
        uint4 w[kChunks];
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            const int64_t c8 = tid + (int64_t)i * kRowThreads;
            w[i] = keys8[c8 < d8 ? c8 : d8 - 1];             // clamped: no load behind a branch
        }
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            const int64_t c8 = tid + (int64_t)i * kRowThreads;
            const bool has = c8 < d8 && max8(w[i]) >= low16;
            const uint32_t at = wave_append(has, &sh.n_words);
            if (has && at < (uint32_t)kWordMax) words[at] = (uint16_t)c8;
        }
    }
    __syncthreads();
    const uint32_t n_words = sh.n_words;
    if (n_words > (uint32_t)kWordMax) {                      // (n_list would overflow as well)
        row_topk<false, false>(s, p, row);
        return;
    }
    for (uint32_t i0 = 0; i0 < n_words; i0 += kRowThreads) {
        const uint32_t i = i0 + tid;
        const uint32_t c8 = words[i < n_words ? i : 0];
        uint32_t k16[8];
        unpack8(keys8[c8], k16);
        uint32_t m = 0u;
#pragma unroll
        for (int t = 0; t < 8; ++t) m |= ((int64_t)c8 * 8 + t < d && k16[t] >= low16) ? (1u << t) : 0u;
        if (i >= n_words) m = 0u;
        const uint32_t mine = (uint32_t)__popc(m);
        const uint32_t incl = wave_inclusive_scan(mine);
        uint32_t base = 0u;
        if (lane == kWave - 1 && incl) base = atomicAdd(&s.ncand, incl);
        uint32_t at = __shfl(base, kWave - 1, kWave) + incl - mine;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (m & (1u << t)) {
                if (at < (uint32_t)kListMax) list[at] = (k16[t] << 16) | (c8 * 8u + t);
                ++at;
            }
        }
    }
    __syncthreads();
    const uint32_t n_list = s.ncand;                         // >= k
    if (n_list > (uint32_t)kListMax) {                       // very many equal magnitudes: the general kernel
        row_topk<false, false>(s, p, row);
        return;
    }

    // ---- 4: the bin of the k-th largest magnitude from the list, narrowed by four more bits if it is crowded
    for (int i = tid; i < (1 << kBits1); i += kRowThreads) s.hist[i] = 0u;     // (held the listed words)
    __syncthreads();
    for (uint32_t i = tid; i < n_list; i += kRowThreads) atomicAdd(&s.hist[list[i] >> (16 + kSubBits)], 1u);
    __syncthreads();
    select_bin(s, 1 << kBits1, k);
    const uint32_t d1 = s.bin;
    uint32_t need = s.need, in_bin = s.hist[d1];
    uint32_t match = d1, match_shift = kSubBits;             // in the bin: prefix >> match_shift == match
    __syncthreads();                                         // hist is free from here on
    if (in_bin > (uint32_t)kCandMax) {
        for (uint32_t i = tid; i < n_list; i += kRowThreads) {
            const uint32_t k16 = list[i] >> 16;
            if ((k16 >> kSubBits) == d1) atomicAdd(&sh.sub[k16 & ((1u << kSubBits) - 1u)], 1u);
        }
        __syncthreads();
        if (tid == 0) {                                      // sixteen counts: one thread walks them from the top
            uint32_t above = 0u;
            for (int sb = (1 << kSubBits) - 1; sb >= 0; --sb) {
                const uint32_t h = sh.sub[sb];
                if (need <= above + h) {
                    s.bin = (uint32_t)sb;
                    s.need = need - above;
                    s.ncand = h;
                    break;
                }
                above += h;
            }
        }
        __syncthreads();
        match = (d1 << kSubBits) | s.bin;
        match_shift = 0;
        need = s.need;
        in_bin = s.ncand;
        __syncthreads();
    }
    if (in_bin > (uint32_t)kCandMax) {                       // still crowded: the general kernel re-reads the row
        row_topk<false, false>(s, p, row);
        return;
    }

    // The bin's entries as 64-bit words key << 16 | (0xffff - position): a larger word goes first in the order
    // (larger key first, lower position first among equal keys).  `kept` collects the positions of the result.
    uint64_t *cand = reinterpret_cast<uint64_t *>(s.hist);               // [kCandMax]
    uint32_t *cand_rank = s.hist + 2 * kCandMax;                        // [kCandMax]
    uint32_t *kept = s.hist + 3 * kCandMax;                             // [kRowThreads]
    if (tid == 0) {
        s.ncand = 0u;
        s.need = 0u;                                         // from here: the number of kept positions
    }
    for (int i = tid; i < kCandMax; i += kRowThreads) cand_rank[i] = 0u;
    __syncthreads();
    for (uint32_t i0 = 0; i0 < n_list; i0 += kRowThreads) {
        const uint32_t i = i0 + tid;
        const uint32_t item = list[i < n_list ? i : 0];
        const uint32_t k16 = item >> 16, e = item & 0xffffu;
        const bool in = i < n_list && (k16 >> match_shift) == match;
        const bool above = i < n_list && (k16 >> match_shift) > match;                 // above the bin: kept
        const uint32_t at_in = wave_append(in, &s.ncand), at_above = wave_append(above, &s.need);
        if (in) cand[at_in] = (uint64_t)e;
        if (above) kept[at_above] = e;
    }
    __syncthreads();
    const uint32_t c = s.ncand;                              // == in_bin >= need >= 1
    for (uint32_t i = tid; i < c; i += kRowThreads) {
        const uint64_t e = cand[i];
        cand[i] = ((uint64_t)mag_key(a[e]) << 16) | (0xffffu - e);
    }
    __syncthreads();
    {
        // c * c comparisons over all threads: thread t compares entry t mod c with one slice of the others
        const uint32_t parts = (uint32_t)kRowThreads / c, per = (c + parts - 1u) / parts;
        if ((uint32_t)tid < c * parts) {
            const uint32_t i = (uint32_t)tid % c, j0 = ((uint32_t)tid / c) * per;
            const uint32_t j1 = j0 + per < c ? j0 + per : c;
            const uint64_t mine = cand[i];
            uint32_t before = 0u;                            // entries that precede this one in the order
            uint32_t j = j0;
            for (; j + 8 <= j1; j += 8) {
                uint64_t other[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) other[u] = cand[j + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) before += other[u] > mine ? 1u : 0u;
            }
            for (; j < j1; ++j) before += cand[j] > mine ? 1u : 0u;
            if (before) atomicAdd(&cand_rank[i], before);
        }
    }
    __syncthreads();
    {                                                        // c <= kCandMax == kRowThreads: one candidate per thread
        const bool keep = (uint32_t)tid < c && cand_rank[tid < (int)c ? tid : 0] < need;
        const uint32_t at = wave_append(keep, &s.need);
        if (keep) kept[at] = 0xffffu - (uint32_t)(cand[tid] & 0xffffu);
    }
    __syncthreads();                                         // s.need == k positions in `kept`, in no order

    // ---- 5: ascending positions.  The kept positions set their bits in a bitmap of the row (in the LDS that held
    // the row, which is done with); an exclusive prefix sum of the bitmap words' bit counts then gives every kept
    // position its place in the output.
    constexpr int kMapWords = (int)(kRow16Max + 31) / 32 + ((int)(kRow16Max + 31) / 32) % 2;   // even
    static_assert(kMapWords <= 2 * kRowThreads, "two bitmap words per thread");
    uint32_t *bitmap = reinterpret_cast<uint32_t *>(keys16);            // [kMapWords]; 8 d >= 8 * kMapWords bytes
    uint32_t *prefix = bitmap + kMapWords;                              // [kMapWords]
    for (int i = tid; i < kMapWords; i += kRowThreads) bitmap[i] = 0u;
    __syncthreads();
    if ((uint32_t)tid < k) atomicOr(&bitmap[kept[tid] >> 5], 1u << (kept[tid] & 31u));
    __syncthreads();
    {
        const uint32_t c0 = 2 * tid < kMapWords ? (uint32_t)__popc(bitmap[2 * tid]) : 0u;
        const uint32_t c1 = 2 * tid + 1 < kMapWords ? (uint32_t)__popc(bitmap[2 * tid + 1]) : 0u;
        const uint32_t incl = wave_inclusive_scan(c0 + c1);
        if (lane == kWave - 1) s.wave_a[tid / kWave] = incl;
        __syncthreads();
        uint32_t run = incl - (c0 + c1);
        for (int v = 0; v < tid / kWave; ++v) run += s.wave_a[v];
        if (2 * tid < kMapWords) prefix[2 * tid] = run;
        if (2 * tid + 1 < kMapWords) prefix[2 * tid + 1] = run + c0;
    }
    __syncthreads();

    // the kept values, read a second time
    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    if ((uint32_t)tid < k) {                                 // k <= 1024: one kept entry per thread
        const uint32_t e = kept[tid];
        const uint32_t at = prefix[e >> 5] + (uint32_t)__popc(bitmap[e >> 5] & ((1u << (e & 31u)) - 1u));
        out_idx[at] = (int32_t)e;
        out_val[at] = a[e];
    }
}

template <bool VEC4>
hipError_t launch(const TopkArgs &p, hipStream_t stream) {
    const size_t dyn = sizeof(uint16_t) * (((size_t)p.d + 7) & ~(size_t)7);
    static PerDeviceOnce configured;           // per instantiation: the attribute belongs to the function
    const hipError_t cfg = configured([] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_row16_kernel<VEC4>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)(sizeof(uint16_t) * (size_t)kRow16Max));
    });
    if (cfg != hipSuccess) return cfg;
    hipLaunchKernelGGL((topk_row16_kernel<VEC4>), dim3((unsigned)p.n), dim3(kRowThreads), dyn, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_topk_row16(const TopkArgs &p, hipStream_t stream) {
    if (p.b || p.g_i || p.parts.part || p.d > kRow16Max || p.d < kRow16Min || p.k > kRow16MaxK)
        return hipErrorInvalidValue;
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0);
    return vec4 ? launch<true>(p, stream) : launch<false>(p, stream);
}

}  // namespace ef21
