// One-workgroup-per-row radix select (Section 2.1 of the EF21 paper: keep the k entries of largest
// magnitude), as device functions shared by the kernels that run it: the stand-alone row kernel
// and the long-row path's per-row select / rescue kernels.  1024 threads per workgroup.
//
// The k largest magnitudes of a row are found on the 31-bit magnitude key (fp32 bits with the sign
// cleared): a histogram pass over the top 12 bits (LDS histogram) finds the bin that holds the k-th largest
// magnitude; the entries of that bin, usually a few dozen, are gathered and ranked against one another
// (two more histogram passes, 10 + 9 bits, when the bin is crowded; no histogram at all for rows of at most
// 256 entries, which are ranked whole), which fixes the key T of the k-th
// largest magnitude and the number q of entries equal to T that are still needed; an ordered
// emission then writes every entry with key > T and the first q entries with key == T, in
// ascending position order (ties go to the lower index).
#pragma once
#include "device_utils.h"
#include "kernels.h"
#include "logreg_finish.h"

namespace ef21 {

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kBits1 = 12, kBits2 = 10, kBits3 = 9;   // 31 key bits
static_assert(kBits1 + kBits2 + kBits3 == 31, "digits must cover the magnitude key");

constexpr int kRankMax = 256;   // a selected bin with at most this many entries is ranked directly

struct RowShared {
    uint32_t hist[1 << kBits1];
    uint32_t wave_a[kRowWaves];
    uint32_t wave_b[kRowWaves];
    uint32_t bin;     // selected digit
    uint32_t need;    // entries still needed from inside the selected bin
    uint32_t ncand;   // entries gathered from the selected bin
    uint32_t cand_key[kRankMax];
    uint32_t cand_idx[kRankMax];
    uint32_t cand_rank[kRankMax];   // low half: gathered entries with a larger key; high half: equal key, lower position
};
static_assert(kRankMax <= 0xffff, "two counts of at most kRankMax share one word");

template <bool DIFF>
__device__ __forceinline__ float load_v(const float *a, const float *b, int64_t e) {
    float v = a[e];
    if (DIFF) v = v - b[e];
    return v;
}

// Histogram of digit ((key >> shift) & (nbins-1)) over the entries whose key >> pshift == prefix.
// value(e) yields entry e of the row.
template <class ValueFn>
__device__ void hist_pass(RowShared &s, int64_t d, ValueFn value, int pshift, uint32_t prefix, int shift, int nbins) {
    for (int i = threadIdx.x; i < nbins; i += kRowThreads) s.hist[i] = 0u;
    __syncthreads();
    const uint32_t mask = (uint32_t)nbins - 1u;
    for (int64_t e = threadIdx.x; e < d; e += kRowThreads) {
        const uint32_t key = mag_key(value(e));
        if ((key >> pshift) == prefix) atomicAdd(&s.hist[(key >> shift) & mask], 1u);
    }
    __syncthreads();
}

// Largest bin b with  count(bins > b) < need <= count(bins >= b).  Leaves b in s.bin and
// need - count(bins > b) in s.need.  Requires need <= total count.
__device__ void select_bin(RowShared &s, int nbins, uint32_t need) {
    const int tid = threadIdx.x;
    const int per = nbins >= kRowThreads ? nbins / kRowThreads : 1;   // bins per thread, from the top
    const int active = nbins / per;
    uint32_t mine = 0u;
    if (tid < active)
        for (int j = 0; j < per; ++j) mine += s.hist[nbins - 1 - (tid * per + j)];
    const uint32_t incl = wave_inclusive_scan(mine);
    const int wave = tid / kWave;
    if (lane_id() == kWave - 1) s.wave_a[wave] = incl;
    __syncthreads();
    uint32_t above = incl - mine;
    for (int w = 0; w < wave; ++w) above += s.wave_a[w];
    if (tid < active && above < need && need <= above + mine) {   // exactly one thread
        uint32_t c = above;
        for (int j = 0; j < per; ++j) {
            const int bin = nbins - 1 - (tid * per + j);
            const uint32_t h = s.hist[bin];
            if (need <= c + h) {
                s.bin = (uint32_t)bin;
                s.need = need - c;
                break;
            }
            c += h;
        }
    }
    __syncthreads();
}

// The entries gathered in s.cand_key / s.cand_idx (s.ncand of them, at most kRankMax, in any order; cand_rank
// zeroed) are ranked against one another in the order "larger key first, lower position first among equal
// keys": c * c comparisons over all threads, thread t comparing entry t mod c with one slice of the others.  The
// entry that need - 1 others precede is the last one kept: its key goes to s.bin (the threshold key T) and the
// number of entries with that key up to and including it to s.need (the tie quota q).  1 <= need <= s.ncand.
__device__ void rank_gathered(RowShared &s, uint32_t need) {
    const uint32_t c = s.ncand;
    const uint32_t parts = (uint32_t)kRowThreads / c, per = (c + parts - 1u) / parts;
    if (threadIdx.x < c * parts) {
        const uint32_t i = threadIdx.x % c, j0 = (threadIdx.x / c) * per;
        const uint32_t j1 = j0 + per < c ? j0 + per : c;
        const uint32_t my_key = s.cand_key[i], my_idx = s.cand_idx[i];
        uint32_t counts = 0u;
#pragma unroll 8
        for (uint32_t j = j0; j < j1; ++j) {
            const uint32_t kj = s.cand_key[j], ij = s.cand_idx[j];
            counts += (kj > my_key ? 1u : 0u) + ((kj == my_key && ij < my_idx) ? 0x10000u : 0u);
        }
        if (counts) atomicAdd(&s.cand_rank[i], counts);
    }
    __syncthreads();
    if (threadIdx.x < c) {
        const uint32_t r = s.cand_rank[threadIdx.x], larger = r & 0xffffu, equal_before = r >> 16;
        if (larger + equal_before == need - 1u) {          // exactly one thread
            s.bin = s.cand_key[threadIdx.x];
            s.need = equal_before + 1u;
        }
    }
    __syncthreads();
}

// Whole Top-k of one row by the calling workgroup (all kRowThreads threads must call).
// value(e) yields entry e of the row (the same bits every time it is asked); with UPDATE the emission
// also applies line 6 of Algorithm 2, g_i[e] = base(e) + value(e), base(e) being the subtracted g_i[e].
template <bool UPDATE, class ValueFn, class BaseFn>
__device__ void row_topk_on(RowShared &s, const TopkArgs &p, int64_t row, ValueFn value, BaseFn base_value) {
    const int64_t d = p.d;

    // ---- threshold key T and tie quota q ------------------------------------------------
    // rows of at most kRankMax entries: every entry is a candidate and the histogram is skipped
    const bool whole_row = d <= kRankMax;
    uint32_t d1 = 0u, need = (uint32_t)p.k, in_bin = (uint32_t)d;
    if (!whole_row) {
        hist_pass(s, d, value, 31, 0u, kBits2 + kBits3, 1 << kBits1);
        select_bin(s, 1 << kBits1, (uint32_t)p.k);
        d1 = s.bin;
        need = s.need;
        in_bin = s.hist[d1];
    }
    if (threadIdx.x == 0) s.ncand = 0u;
    if (threadIdx.x < kRankMax) s.cand_rank[threadIdx.x] = 0u;
    __syncthreads();                             // everybody has read hist[d1] before either branch reuses hist
    uint32_t T, q;
    if (in_bin <= (uint32_t)kRankMax) {
        // the bin's entries side by side (in any order), then every one counts those that go before it in the
        // order (larger key first, lower position first among equal keys): the one that `need - 1` others
        // precede is the last entry kept, its key is T, and q counts it and the equal keys before it
        for (int64_t e = threadIdx.x; e < d; e += kRowThreads) {
            const uint32_t key = mag_key(value(e));
            if (whole_row || (key >> (kBits2 + kBits3)) == d1) {
                const uint32_t at = atomicAdd(&s.ncand, 1u);
                s.cand_key[at] = key;
                s.cand_idx[at] = (uint32_t)e;
            }
        }
        __syncthreads();
        rank_gathered(s, need);
        T = s.bin;
        q = s.need;
    } else {
        hist_pass(s, d, value, kBits2 + kBits3, d1, kBits3, 1 << kBits2);
        select_bin(s, 1 << kBits2, need);
        const uint32_t d12 = (d1 << kBits2) | s.bin;
        need = s.need;
        hist_pass(s, d, value, kBits3, d12, 0, 1 << kBits3);
        select_bin(s, 1 << kBits3, need);
        T = (d12 << kBits3) | s.bin;
        q = s.need;   // 1 <= q <= number of entries with key == T
    }

    // ---- ordered emission: each wavefront owns a contiguous piece of the row -------------
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    int64_t piece = (d + kRowWaves - 1) / kRowWaves;
    piece = (piece + kWave - 1) / kWave * kWave;
    const int64_t lo = wave * piece < d ? wave * piece : d;
    const int64_t hi = lo + piece < d ? lo + piece : d;

    uint32_t n_gt = 0u, n_eq = 0u;
    for (int64_t base = lo; base < hi; base += kWave) {
        const int64_t e = base + lane;
        uint32_t key = 0u;
        const bool in = e < hi;
        if (in) key = mag_key(value(e));
        n_gt += popc64(__ballot(in && key > T));
        n_eq += popc64(__ballot(in && key == T));
    }
    if (lane == 0) {
        s.wave_a[wave] = n_gt;
        s.wave_b[wave] = n_eq;
    }
    __syncthreads();
    uint32_t gt_before = 0u, eq_run = 0u;
    for (int w = 0; w < wave; ++w) {
        gt_before += s.wave_a[w];
        eq_run += s.wave_b[w];
    }
    uint32_t out_run = gt_before + (eq_run < q ? eq_run : q);

    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    float *g_i = UPDATE ? p.g_i + row * d : nullptr;
    for (int64_t base = lo; base < hi; base += kWave) {
        const int64_t e = base + lane;
        const bool in = e < hi;
        const float v = in ? value(e) : 0.f;
        const uint32_t key = mag_key(v);
        const bool gt = in && key > T;
        const bool eq = in && key == T;
        const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
        const uint32_t eq_below = eq_run + lanes_below(m_eq);   // ties before this lane, whole row
        const uint32_t ties_taken_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
        const bool keep = gt || (eq && eq_below < q);
        if (keep) {
            const uint32_t pos = out_run + lanes_below(m_gt) + ties_taken_before;
            out_idx[pos] = (int32_t)e;
            out_val[pos] = v;
            if (UPDATE) g_i[e] = base_value(e) + v;    // Algorithm 2, line 6
        }
        const uint32_t eq_next = eq_run + popc64(m_eq);
        out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_run < q ? eq_run : q));
        eq_run = eq_next;
    }
}

// The row read from global memory in every pass (any d).
template <bool DIFF, bool UPDATE>
__device__ void row_topk(RowShared &s, const TopkArgs &p, int64_t row) {
    const float *a = p.a + row * p.d;
    const float *b = DIFF ? p.b + row * p.d : nullptr;
    row_topk_on<UPDATE>(
        s, p, row, [=](int64_t e) { return load_v<DIFF>(a, b, e); }, [=](int64_t e) { return DIFF ? b[e] : 0.f; });
}

// Rows of at most kRowCache entries: the row is formed once into LDS (`cache`), all passes read it there.
constexpr int kRowCache = 8192;

template <bool DIFF, bool UPDATE>
__device__ void row_topk_cached(RowShared &s, float *cache, const TopkArgs &p, int64_t row) {
    const int64_t d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    for (int64_t e = threadIdx.x; e < d; e += kRowThreads) cache[e] = load_v<DIFF>(a, b, e);
    __syncthreads();
    row_topk_on<UPDATE>(
        s, p, row, [=](int64_t e) { return cache[e]; }, [=](int64_t e) { return DIFF ? b[e] : 0.f; });
}

// Same, the row being grad f_i - g_i with the gradient still in partial sums (p.parts).
template <bool UPDATE>
__device__ void row_topk_parts(RowShared &s, float *cache, const TopkArgs &p, int64_t row) {
    const int64_t d = p.d;
    const float *part_w = p.parts.part + row * p.parts.chunks * d;
    const float *b = p.b + row * d;
    for (int64_t e = threadIdx.x; e < d; e += kRowThreads)
        cache[e] = dense_grad_entry(part_w, p.parts.chunks, d, e, p.parts.x[e], p.parts.m, p.parts.lambda) - b[e];
    __syncthreads();
    row_topk_on<UPDATE>(
        s, p, row, [=](int64_t e) { return cache[e]; }, [=](int64_t e) { return b[e]; });
}

}  // namespace ef21
