// Batched Top-k (Section 2.1 of the EF21 paper) for long rows: many workgroups per row, the row
// itself read ONCE.
//
// Same selection rule as the one-workgroup kernel (31-bit magnitude key, ties to the lower index,
// ascending output).  Pipeline:
//
//   collect   Every workgroup first looks at the same fixed sample of its row (64 evenly spaced
//             pieces of 256 entries), finds in LDS a key `key_lo` that, with overwhelming
//             probability, at least k entries of the row reach, and then streams its part of the
//             row.  Each wavefront owns a contiguous piece of the row and appends the entries
//             with key >= key_lo ("candidates", a few per cent of the row) in position order to
//             its own slot of the workspace.  No atomics, no fences, no inter-workgroup traffic.
//   then, on the candidates only, either
//   select    (small k) one workgroup per row: candidate keys into LDS, radix select there, ordered
//             emission of the k kept entries (+ lines 6 and 8 of Algorithm 2); or
//   hist x3, count, emit, rescue   (large k) the same steps spread over 16 workgroups per row,
//             chained by kernel boundaries: a kernel merges its LDS histograms into the row's
//             global one with a few atomics per bin, the NEXT kernel's workgroups each scan the
//             merged histogram in their prologue.
//
// The estimate can be wrong (fewer than k candidates); the row is then selected by the exact
// one-workgroup algorithm on the original data (inside `select`, or by `rescue`), so the result
// never depends on the sample.  Slots have the capacity of their piece, so any input fits.
#include <cmath>

#include "topk_row_impl.h"

namespace ef21 {
namespace {

constexpr int kBlk = kRowThreads;            // collect / select / rescue workgroups
constexpr int kBlkWaves = kBlk / kWave;
constexpr int kSample = 16384;               // sampled entries per row
constexpr int kSamplePer = kSample / kBlk;
constexpr int kPieceLen = 256, kPieces = kSample / kPieceLen;
constexpr int kMaxSlots = 4096;              // slots (wavefront pieces) per row
constexpr int kSelCap = 28672;               // candidate keys the select kernel holds in LDS
constexpr int kCandThreads = 256;            // candidate-stage workgroups (large k)
constexpr int kCandWaves = kCandThreads / kWave;
constexpr int kCandBlocks = 16;              // per row: 64 wavefronts, one slot each per round
constexpr int kBins1 = 1 << kBits1, kBins2 = 1 << kBits2, kBins3 = 1 << kBits3;

struct RowInfo {
    uint32_t failed, M;   // fewer than k candidates were collected; number of candidates
    uint32_t d1, need1;   // first digit of the threshold key; entries still needed from that bin
    uint32_t p22, need2;  // first two digits; entries still needed from that sub-bin
    uint32_t T, q;        // threshold key; number of entries equal to T to keep
};

struct Ws {
    uint32_t *hist1, *hist2, *hist3;      // [n][bins], kept zero between calls
    RowInfo *info;                        // [n]
    uint32_t *slot_cnt, *slot_gt, *slot_eq;   // [n][nslot]
    int32_t *cand_idx;                    // [n][nslot][L]
    float *cand_val;
    int64_t L;                            // entries per wavefront piece = slot capacity
    int64_t nslot;                        // pieces per row
    int64_t G;                            // collect workgroups per row
};

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

void plan(int32_t n, int64_t d, Ws *w) {
    int64_t max_g = 512 / n;                                  // about two 1024-thread workgroups per CU
    if (max_g < 1) max_g = 1;
    if (max_g > kMaxSlots / kBlkWaves) max_g = kMaxSlots / kBlkWaves;
    int64_t g = (d + kBlkWaves * 2048 - 1) / (kBlkWaves * 2048);   // at least 2048 entries per piece
    if (g > max_g) g = max_g;
    if (g < 1) g = 1;
    const int64_t pieces = g * kBlkWaves;
    int64_t L = (d + pieces - 1) / pieces;
    L = (L + 255) / 256 * 256;
    w->L = L;
    w->nslot = (d + L - 1) / L;
    w->G = (w->nslot + kBlkWaves - 1) / kBlkWaves;
}

size_t layout(int32_t n, int64_t d, char *base, Ws *w) {
    Ws tmp;
    plan(n, d, &tmp);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += align256(bytes);
        return p;
    };
    char *h1 = take(sizeof(uint32_t) * (size_t)n * kBins1);
    char *h2 = take(sizeof(uint32_t) * (size_t)n * kBins2);
    char *h3 = take(sizeof(uint32_t) * (size_t)n * kBins3);
    char *inf = take(sizeof(RowInfo) * (size_t)n);
    const size_t slots = sizeof(uint32_t) * (size_t)n * tmp.nslot;
    char *s0 = take(slots), *s1 = take(slots), *s2 = take(slots);
    char *ci = take(sizeof(int32_t) * (size_t)n * tmp.nslot * tmp.L);
    char *cv = take(sizeof(float) * (size_t)n * tmp.nslot * tmp.L);
    if (w) {
        *w = tmp;
        w->hist1 = (uint32_t *)h1; w->hist2 = (uint32_t *)h2; w->hist3 = (uint32_t *)h3;
        w->info = (RowInfo *)inf;
        w->slot_cnt = (uint32_t *)s0; w->slot_gt = (uint32_t *)s1; w->slot_eq = (uint32_t *)s2;
        w->cand_idx = (int32_t *)ci; w->cand_val = (float *)cv;
    }
    return off;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// ---------------------------------------------------------------- collect
// Sample rank r such that the r-th largest sampled key is, except with negligible probability,
// not above the k-th largest key of the row: mean + 5 standard deviations + 8 of the number of
// sampled entries among the row's top k (a binomial with mean mu = k * sample / d).
__device__ __forceinline__ uint32_t sample_rank(int64_t k, int64_t ns, int64_t d) {
    if (ns >= d) return (uint32_t)k;      // the sample is the row
    const double mu = (double)k * (double)ns / (double)d;
    return (uint32_t)ceil(mu + 5.0 * sqrt(mu) + 8.0);
}

// Lower bound of the candidate keys, identical in every workgroup of a row (it depends on the data
// only).  22 significant bits; 0 means "every entry is a candidate".
template <bool DIFF>
__device__ uint32_t estimate_key_lo(RowShared &s, const float *a, const float *b, int64_t d, int64_t k) {
    const int64_t ns = d < kSample ? d : kSample;
    const uint32_t r = sample_rank(k, ns, d);
    if (r > ns) return 0u;
    uint32_t skey[kSamplePer];
#pragma unroll
    for (int j = 0; j < kSamplePer; ++j) {
        const int64_t i = threadIdx.x + (int64_t)j * kBlk;
        skey[j] = 0xffffffffu;            // marks "no sample" (a magnitude key has bit 31 clear)
        if (i < ns) {
            int64_t e = i;
            if (d > kSample) e = ((i / kPieceLen) * (d - kPieceLen)) / (kPieces - 1) + (i % kPieceLen);
            skey[j] = mag_key(load_v<DIFF>(a, b, e));
        }
    }
    for (int i = threadIdx.x; i < kBins1; i += kBlk) s.hist[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSamplePer; ++j)
        if (skey[j] != 0xffffffffu) atomicAdd(&s.hist[skey[j] >> (kBits2 + kBits3)], 1u);
    __syncthreads();
    select_bin(s, kBins1, r);
    const uint32_t d1 = s.bin, r1 = s.need;
    __syncthreads();
    for (int i = threadIdx.x; i < kBins2; i += kBlk) s.hist[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kSamplePer; ++j)
        if (skey[j] != 0xffffffffu && (skey[j] >> (kBits2 + kBits3)) == d1)
            atomicAdd(&s.hist[(skey[j] >> kBits3) & (kBins2 - 1)], 1u);
    __syncthreads();
    select_bin(s, kBins2, r1);
    const uint32_t key_lo = ((d1 << kBits2) | s.bin) << kBits3;
    __syncthreads();
    return key_lo;
}

// A wavefront walks its piece in steps of 64*VEC entries.  VEC = 4 needs 16-byte aligned rows.
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
                    const float4 u = *reinterpret_cast<const float4 *>(b + e0);
                    v[0] -= u.x; v[1] -= u.y; v[2] -= u.z; v[3] -= u.w;
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

template <int VEC, bool DIFF>
__global__ __launch_bounds__(kBlk) void split_collect_kernel(TopkArgs p, Ws w) {
    __shared__ RowShared s;
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    const uint32_t key_lo = estimate_key_lo<DIFF>(s, a, b, d, p.k);

    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t slot = (int64_t)blockIdx.x * kBlkWaves + wave;
    if (slot >= w.nslot) return;
    const int64_t lo = slot * w.L;
    const int64_t hi = lo + w.L < d ? lo + w.L : d;
    int32_t *slot_idx = w.cand_idx + (row * w.nslot + slot) * w.L;
    float *slot_val = w.cand_val + (row * w.nslot + slot) * w.L;
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
                c[t] = (e0 + t < hi) && mag_key(st[u].v[t]) >= key_lo;
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
                        ++pos;
                    }
                }
                cnt += all;
            }
        }
    }
    if (lane == 0) w.slot_cnt[row * w.nslot + slot] = cnt;
}

// ---------------------------------------------------------------- select (small k): one workgroup per row
template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kBlk) void split_select_kernel(TopkArgs p, Ws w) {
    __shared__ RowShared s;
    __shared__ uint32_t off[kMaxSlots + 1];      // exclusive prefix of the slot counts
    extern __shared__ uint32_t keys[];           // [kSelCap]
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    const int nslot = (int)w.nslot;
    const uint32_t *slot_cnt = w.slot_cnt + row * w.nslot;

    // exclusive scan of the slot counts: four consecutive slots per thread
    constexpr int kPer = kMaxSlots / kBlk;
    uint32_t c[kPer], mine = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int sl = tid * kPer + j;
        c[j] = sl < nslot ? slot_cnt[sl] : 0u;
        mine += c[j];
    }
    const uint32_t incl = wave_inclusive_scan(mine);
    if (lane == kWave - 1) s.wave_a[wave] = incl;
    __syncthreads();
    uint32_t run = incl - mine;
    for (int v = 0; v < wave; ++v) run += s.wave_a[v];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int sl = tid * kPer + j;
        off[sl] = run;
        run += c[j];
    }
    if (tid == kBlk - 1) off[kMaxSlots] = run;   // slots beyond nslot count as empty, so off[nslot] = M
    __syncthreads();
    const uint32_t M = off[nslot];
    if (M < (uint32_t)p.k || M > (uint32_t)kSelCap) {    // estimate failed, or too many candidates for LDS
        row_topk<DIFF, UPDATE>(s, p, row);
        return;
    }

    // slot of flat candidate j: the last slot whose prefix is <= j
    auto slot_of = [&](uint32_t j) {
        int lo = 0, hi = nslot;                  // invariant: off[lo] <= j < off[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (off[mid] <= j) lo = mid;
            else hi = mid;
        }
        return lo;
    };
    const float *cand_val = w.cand_val + row * w.nslot * w.L;
    const int32_t *cand_idx = w.cand_idx + row * w.nslot * w.L;
    for (uint32_t j = tid; j < M; j += kBlk) {
        const int sl = slot_of(j);
        keys[j] = mag_key(cand_val[(int64_t)sl * w.L + (j - off[sl])]);
    }
    __syncthreads();

    // radix select over the keys in LDS
    uint32_t prefix = 0, need = (uint32_t)p.k;
    {
        const int shifts[3] = {kBits2 + kBits3, kBits3, 0};
        const int pshifts[3] = {31, kBits2 + kBits3, kBits3};
        const int bins[3] = {kBins1, kBins2, kBins3};
        for (int pass = 0; pass < 3; ++pass) {
            for (int i = tid; i < bins[pass]; i += kBlk) s.hist[i] = 0u;
            __syncthreads();
            for (uint32_t j = tid; j < M; j += kBlk) {
                const uint32_t key = keys[j];
                if ((key >> pshifts[pass]) == prefix) atomicAdd(&s.hist[(key >> shifts[pass]) & (bins[pass] - 1)], 1u);
            }
            __syncthreads();
            select_bin(s, bins[pass], need);
            prefix = (prefix << (pass == 0 ? 0 : (pass == 1 ? kBits2 : kBits3))) | s.bin;
            need = s.need;
            __syncthreads();
        }
    }
    const uint32_t T = prefix, q = need;

    // ordered emission: each wavefront owns a contiguous range of the flat candidate list
    uint32_t piece = (M + kBlkWaves - 1) / kBlkWaves;
    piece = (piece + kWave - 1) / kWave * kWave;
    const uint32_t lo = (uint32_t)wave * piece < M ? (uint32_t)wave * piece : M;
    const uint32_t hi = lo + piece < M ? lo + piece : M;
    uint32_t n_gt = 0, n_eq = 0;
    for (uint32_t base = lo; base < hi; base += kWave) {
        const uint32_t j = base + lane;
        const uint32_t key = j < hi ? keys[j] : 0u;
        n_gt += popc64(__ballot(j < hi && key > T));
        n_eq += popc64(__ballot(j < hi && key == T));
    }
    if (lane == 0) {
        s.wave_a[wave] = n_gt;
        s.wave_b[wave] = n_eq;
    }
    __syncthreads();
    uint32_t gt_before = 0, eq_run = 0;
    for (int v = 0; v < wave; ++v) {
        gt_before += s.wave_a[v];
        eq_run += s.wave_b[v];
    }
    uint32_t out_run = gt_before + (eq_run < q ? eq_run : q);
    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    for (uint32_t base = lo; base < hi; base += kWave) {
        const uint32_t j = base + lane;
        const bool in = j < hi;
        const uint32_t key = in ? keys[j] : 0u;
        const bool gt = in && key > T, eq = in && key == T;
        const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
        const uint32_t eq_below = eq_run + lanes_below(m_eq);
        const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
        if (gt || (eq && eq_below < q)) {
            const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
            const int sl = slot_of(j);
            const int64_t at = (int64_t)sl * w.L + (j - off[sl]);
            const int32_t e = cand_idx[at];
            const float v = cand_val[at];
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

// ---------------------------------------------------------------- candidate stages (large k)
// exclusive prefix sum over the workgroup's threads; total returned through *total
__device__ uint32_t cand_block_scan(uint32_t v, uint32_t *lds_wave /*[kCandWaves]*/, uint32_t *total) {
    const uint32_t incl = wave_inclusive_scan(v);
    const int wave = threadIdx.x / kWave;
    __syncthreads();                       // lds_wave may still be in use by a previous scan
    if (lane_id() == kWave - 1) lds_wave[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (int v2 = 0; v2 < kCandWaves; ++v2) {
        const uint32_t t = lds_wave[v2];
        if (v2 < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// Digit selection over the row's merged histogram (written by the previous kernel): largest bin b
// with count(bins > b) < need <= count(bins >= b).  lds_out[0] = b, lds_out[1] = need - count(bins > b).
template <int NBINS>
__device__ void select_digit(const uint32_t *hist, uint32_t need, uint32_t *lds_wave, uint32_t *lds_out) {
    constexpr int PER = NBINS / kCandThreads;      // bins per thread, walked from the top
    static_assert(PER >= 1 && PER * kCandThreads == NBINS, "histogram size must be a multiple of the workgroup");
    uint32_t h[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[j] = hist[NBINS - 1 - ((int)threadIdx.x * PER + j)];
        mine += h[j];
    }
    uint32_t total;
    const uint32_t above = cand_block_scan(mine, lds_wave, &total);
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

template <int NBINS>
__device__ void zero_lds_hist(uint32_t *hist) {
    for (int i = threadIdx.x; i < NBINS; i += kCandThreads) hist[i] = 0u;
    __syncthreads();
}

// Adds a workgroup's LDS histogram into the row's global one (non-empty bins only).
template <int NBINS>
__device__ void flush_hist(const uint32_t *lds_hist, uint32_t *global_hist) {
    __syncthreads();
    for (int b = threadIdx.x; b < NBINS; b += kCandThreads) {
        const uint32_t c = lds_hist[b];
        if (c) atomicAdd(global_hist + b, c);
    }
}

__device__ void zero_global_hist(uint32_t *hist, int bins) {
    for (int i = threadIdx.x; i < bins; i += kCandThreads) hist[i] = 0u;
}

// Digit STAGE (1, 2 or 3) of the radix select over the candidates.  Prologue: the result of the
// previous stage from the merged histogram; body: histogram of this stage's digit.
template <int STAGE>
__global__ __launch_bounds__(kCandThreads) void cand_hist_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t hist[STAGE == 1 ? kBins1 : (STAGE == 2 ? kBins2 : kBins3)];
    __shared__ uint32_t lds_wave[kCandWaves], lds_out[2];
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    const uint32_t *slot_cnt = w.slot_cnt + row * w.nslot;
    uint32_t prefix = 0;    // digits known so far
    if constexpr (STAGE == 1) {
        uint32_t mine = 0, M;
        for (int64_t sl = threadIdx.x; sl < w.nslot; sl += kCandThreads) mine += slot_cnt[sl];
        (void)cand_block_scan(mine, lds_wave, &M);
        const bool failed = M < (uint32_t)p.k;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            info->failed = failed ? 1u : 0u;
            info->M = M;
        }
        if (failed) return;
    } else {
        if (info->failed) return;
        if constexpr (STAGE == 2) {
            select_digit<kBins1>(w.hist1 + row * kBins1, (uint32_t)p.k, lds_wave, lds_out);
            prefix = lds_out[0];
            if (blockIdx.x == 0 && threadIdx.x == 0) {
                info->d1 = lds_out[0];
                info->need1 = lds_out[1];
            }
        } else {
            select_digit<kBins2>(w.hist2 + row * kBins2, info->need1, lds_wave, lds_out);
            prefix = (info->d1 << kBits2) | lds_out[0];
            if (blockIdx.x == 0 && threadIdx.x == 0) {
                info->p22 = prefix;
                info->need2 = lds_out[1];
            }
            if (blockIdx.x == 0) zero_global_hist(w.hist1 + row * kBins1, kBins1);   // consumed by stage 2
        }
    }
    constexpr int NB = STAGE == 1 ? kBins1 : (STAGE == 2 ? kBins2 : kBins3);
    constexpr int SHIFT = STAGE == 1 ? kBits2 + kBits3 : (STAGE == 2 ? kBits3 : 0);
    constexpr int PSHIFT = STAGE == 1 ? 31 : (STAGE == 2 ? kBits2 + kBits3 : kBits3);
    zero_lds_hist<NB>(hist);
    for (int64_t sl = (int64_t)blockIdx.x * kCandWaves + wave; sl < w.nslot; sl += kCandBlocks * kCandWaves) {
        const uint32_t cnt = slot_cnt[sl];
        const float *slot_val = w.cand_val + (row * w.nslot + sl) * w.L;
        for (uint32_t j = lane; j < cnt; j += kWave) {
            const uint32_t key = mag_key(slot_val[j]);
            if ((key >> PSHIFT) == prefix) atomicAdd(&hist[(key >> SHIFT) & (NB - 1)], 1u);
        }
    }
    uint32_t *merged = STAGE == 1 ? w.hist1 + row * kBins1 : (STAGE == 2 ? w.hist2 + row * kBins2 : w.hist3 + row * kBins3);
    flush_hist<NB>(hist, merged);
}

// Prologue: threshold key T and tie quota q from the third digit's histogram.  Body: per slot, the
// number of candidates above T and equal to T.
__global__ __launch_bounds__(kCandThreads) void cand_count_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t lds_wave[kCandWaves], lds_out[2];
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    if (info->failed) return;
    select_digit<kBins3>(w.hist3 + row * kBins3, info->need2, lds_wave, lds_out);
    const uint32_t T = (info->p22 << kBits3) | lds_out[0];
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            info->T = T;
            info->q = lds_out[1];
        }
        zero_global_hist(w.hist2 + row * kBins2, kBins2);     // consumed by stage 3
    }
    for (int64_t sl = (int64_t)blockIdx.x * kCandWaves + wave; sl < w.nslot; sl += kCandBlocks * kCandWaves) {
        const uint32_t cnt = w.slot_cnt[row * w.nslot + sl];
        const float *slot_val = w.cand_val + (row * w.nslot + sl) * w.L;
        uint32_t n_gt = 0, n_eq = 0;
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const uint32_t j = j0 + lane;
            const uint32_t key = j < cnt ? mag_key(slot_val[j]) : 0u;
            n_gt += popc64(__ballot(j < cnt && key > T));
            n_eq += popc64(__ballot(j < cnt && key == T));
        }
        if (lane == 0) {
            w.slot_gt[row * w.nslot + sl] = n_gt;
            w.slot_eq[row * w.nslot + sl] = n_eq;
        }
    }
    (void)p;
}

// Ordered emission.  A wavefront handles slots sl, sl + 64, sl + 128, ... and carries the number of
// kept entries and of ties in all earlier slots along, 64 slot counts per round.
template <bool UPDATE>
__global__ __launch_bounds__(kCandThreads) void cand_emit_kernel(TopkArgs p, Ws w) {
    static_assert(kCandBlocks * kCandWaves == kWave, "a wavefront advances by one lane-width of slots per round");
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const RowInfo *info = w.info + row;
    if (info->failed) return;
    if (blockIdx.x == 0) zero_global_hist(w.hist3 + row * kBins3, kBins3);       // consumed by count
    const uint32_t T = info->T, q = info->q;
    const uint32_t *slot_gt = w.slot_gt + row * w.nslot, *slot_eq = w.slot_eq + row * w.nslot;
    const int64_t first = (int64_t)blockIdx.x * kCandWaves + wave;              // < 64
    uint32_t gt_run = wave_sum_u32(lane < first && lane < w.nslot ? slot_gt[lane] : 0u);
    uint32_t eq_run = wave_sum_u32(lane < first && lane < w.nslot ? slot_eq[lane] : 0u);
    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    for (int64_t sl = first; sl < w.nslot; sl += kWave) {
        const uint32_t cnt = w.slot_cnt[row * w.nslot + sl];
        const int32_t *slot_idx = w.cand_idx + (row * w.nslot + sl) * w.L;
        const float *slot_val = w.cand_val + (row * w.nslot + sl) * w.L;
        uint32_t out_run = gt_run + (eq_run < q ? eq_run : q);
        uint32_t eq_in = eq_run;
        for (uint32_t j0 = 0; j0 < cnt; j0 += kWave) {
            const uint32_t j = j0 + lane;
            const bool in = j < cnt;
            const float v = in ? slot_val[j] : 0.f;
            const uint32_t key = mag_key(v);
            const bool gt = in && key > T, eq = in && key == T;
            const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
            const uint32_t eq_below = eq_in + lanes_below(m_eq);
            const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_in < q ? eq_in : q);
            if (gt || (eq && eq_below < q)) {
                const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
                const int32_t e = slot_idx[j];
                out_idx[pos] = e;
                out_val[pos] = v;
                if (UPDATE) {
                    float *g_i = p.g_i + row * p.d;
                    g_i[e] = g_i[e] + v;                   // Algorithm 2, line 6
                    atomicAdd(p.g + e, v * p.inv_n);       // Algorithm 2, line 8
                }
            }
            const uint32_t eq_next = eq_in + popc64(m_eq);
            out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_in < q ? eq_in : q));
            eq_in = eq_next;
        }
        // advance the running counts over slots sl .. sl+63
        const int64_t t = sl + lane;
        gt_run += wave_sum_u32(t < w.nslot ? slot_gt[t] : 0u);
        eq_run += wave_sum_u32(t < w.nslot ? slot_eq[t] : 0u);
    }
}

// Rows whose estimate failed are selected by the exact one-workgroup algorithm.
template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kBlk) void split_rescue_kernel(TopkArgs p, Ws w) {
    __shared__ RowShared s;
    if (!w.info[blockIdx.x].failed) return;
    row_topk<DIFF, UPDATE>(s, p, blockIdx.x);
}

__global__ __launch_bounds__(kCandThreads) void zero_words_kernel(uint32_t *p, size_t words) {
    const size_t stride = (size_t)gridDim.x * kCandThreads;
    for (size_t i = (size_t)blockIdx.x * kCandThreads + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

template <int VEC, bool DIFF>
void launch_collect(const TopkArgs &p, const Ws &w, hipStream_t stream) {
    hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF>), dim3((unsigned)w.G, (unsigned)p.n), dim3(kBlk), 0, stream, p,
                       w);
}

template <bool DIFF, bool UPDATE>
hipError_t launch_select(const TopkArgs &p, const Ws &w, hipStream_t stream) {
    constexpr size_t kDyn = sizeof(uint32_t) * kSelCap;
    static bool configured = false;    // per instantiation; the attribute is a property of the function
    if (!configured) {
        hipError_t st = hipFuncSetAttribute(reinterpret_cast<const void *>(&split_select_kernel<DIFF, UPDATE>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDyn);
        if (st != hipSuccess) return st;
        configured = true;
    }
    hipLaunchKernelGGL((split_select_kernel<DIFF, UPDATE>), dim3((unsigned)p.n), dim3(kBlk), kDyn, stream, p, w);
    return hipGetLastError();
}

// candidates the collect pass is expected to keep per row (see sample_rank)
double expected_candidates(int64_t d, int64_t k) {
    const double ns = d < kSample ? (double)d : (double)kSample;
    const double mu = (double)k * ns / (double)d;
    return (mu + 5.0 * std::sqrt(mu) + 8.0) * (double)d / ns * 1.1;
}

}  // namespace

size_t topk_split_workspace_bytes(int32_t n, int64_t d, int64_t) { return layout(n, d, nullptr, nullptr); }

hipError_t launch_topk_split_reset(void *workspace, int32_t n, int64_t d, hipStream_t stream) {
    Ws w;
    layout(n, d, (char *)workspace, &w);
    // the histograms are the leading, contiguous part of the layout
    const size_t words = ((char *)w.info - (char *)workspace) / sizeof(uint32_t);
    size_t blocks = (words + kCandThreads - 1) / kCandThreads;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(kCandThreads), 0, stream, (uint32_t *)workspace,
                       words);
    return hipGetLastError();
}

hipError_t launch_topk_split(const TopkArgs &p, void *workspace, hipStream_t stream, const Marker &mk) {
    Ws w;
    layout(p.n, p.d, (char *)workspace, &w);
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    if (upd && !diff) return hipErrorInvalidValue;
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0) && (!diff || (uintptr_t)p.b % 16 == 0);
    if (vec4 && diff) launch_collect<4, true>(p, w, stream);
    else if (vec4) launch_collect<4, false>(p, w, stream);
    else if (diff) launch_collect<1, true>(p, w, stream);
    else launch_collect<1, false>(p, w, stream);
    mk(K_TOPK_COLLECT);
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return st;

    if (expected_candidates(p.d, p.k) <= (double)kSelCap) {
        if (upd) st = launch_select<true, true>(p, w, stream);
        else if (diff) st = launch_select<true, false>(p, w, stream);
        else st = launch_select<false, false>(p, w, stream);
        mk(K_TOPK_SELECT);
        return st;
    }
    const dim3 grid(kCandBlocks, (unsigned)p.n), block(kCandThreads);
    hipLaunchKernelGGL(cand_hist_kernel<1>, grid, block, 0, stream, p, w);
    mk(K_TOPK_REFINE);
    hipLaunchKernelGGL(cand_hist_kernel<2>, grid, block, 0, stream, p, w);
    mk(K_TOPK_REFINE);
    hipLaunchKernelGGL(cand_hist_kernel<3>, grid, block, 0, stream, p, w);
    mk(K_TOPK_REFINE);
    hipLaunchKernelGGL(cand_count_kernel, grid, block, 0, stream, p, w);
    mk(K_TOPK_COUNT);
    if (upd) hipLaunchKernelGGL(cand_emit_kernel<true>, grid, block, 0, stream, p, w);
    else hipLaunchKernelGGL(cand_emit_kernel<false>, grid, block, 0, stream, p, w);
    mk(K_TOPK_EMIT);
    if (upd) hipLaunchKernelGGL((split_rescue_kernel<true, true>), dim3((unsigned)p.n), dim3(kBlk), 0, stream, p, w);
    else if (diff) hipLaunchKernelGGL((split_rescue_kernel<true, false>), dim3((unsigned)p.n), dim3(kBlk), 0, stream, p, w);
    else hipLaunchKernelGGL((split_rescue_kernel<false, false>), dim3((unsigned)p.n), dim3(kBlk), 0, stream, p, w);
    mk(K_TOPK_ROW);
    return hipGetLastError();
}

}  // namespace ef21
