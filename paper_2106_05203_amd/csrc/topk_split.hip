// Batched Top-k (Section 2.1 of the EF21 paper) for long rows: many workgroups per row, the row
// itself read ONCE.
//
// Same selection rule as the one-workgroup kernel (31-bit magnitude key, ties to the lower index,
// ascending output).  Three kernels:
//
//   collect   A key `key_lo` that (almost surely) at least k entries of the row reach is fixed first: from the
//             threshold key T of the previous call on the same quantity, lowered by a few per cent (warm start:
//             inside ef21_step consecutive iterations select nearly the same T), else from a fixed sample of the
//             row (64 evenly spaced pieces of 64 entries) that every workgroup of the row looks at.  Then each
//             wavefront streams a contiguous piece of the row and appends the entries with key >= key_lo
//             ("candidates", one or two per cent of the row) in position order to its own slot of the workspace,
//             counting them into the workgroup's LDS histogram of (key - key_lo) >> shift on the way (4096 bins;
//             keys beyond the window share the last bin).  The workgroup's histogram is added to the row's with
//             one atomic per non-empty bin.  No fences, no waiting.
//   count     Prologue of every workgroup: the bin that holds T, from the row's histogram.  Body, one wavefront
//             per slot: the slot's number of candidates in higher bins, and the candidates of T's bin (a handful)
//             appended to the row's short "tie list".
//   emit      Prologue: the tie list ranked in LDS (larger key first, lower position first) gives T and the number
//             q of entries equal to T to keep; the counts of the earlier slots give the output offset.  Body, one
//             wavefront per slot: ordered emission of the k kept entries (+ line 6 of Algorithm 2 on request).
//
// The guess can be wrong: fewer than k candidates, T beyond the histogram's window, or a crowded bin (more
// than kTieCap entries, i.e. very many equal magnitudes at the threshold).  After a warm start a second collect
// pass (normally a launch that ends at once) redoes such a row from the sample; a row that still fails is selected
// by the exact one-workgroup algorithm on the original data (an extra workgroup of the count kernel), so the
// result never depends on the guess.  Slots have the capacity of their piece, so any input fits.
#include <algorithm>
#include <cmath>

#include "topk_row_impl.h"

namespace ef21 {
namespace {

constexpr int kBlk = kRowThreads;            // collect / rescue workgroups
constexpr int kBlkWaves = kBlk / kWave;
constexpr int kSample = 4096;                // sampled entries per row
constexpr int kSamplePer = kSample / kBlk;
constexpr int kPieceLen = 64, kPieces = kSample / kPieceLen;   // a wavefront's load is one piece
constexpr int kMaxSlots = 4096;              // slots (wavefront pieces) per row
constexpr int kCandThreads = 1024;           // count / emit workgroups: one wavefront per slot
constexpr int kCandWaves = kCandThreads / kWave;
constexpr int kBins1 = 1 << kBits1;
constexpr int kHistBins = 4096;              // bins of the candidates' histogram
static_assert(kHistBins == kBins1, "the candidates' histogram lives in RowShared::hist");
static_assert(kCandThreads == kRowThreads && kBlk == kRowThreads, "the rescue runs the one-workgroup algorithm");
// Bin width of the candidates' histogram as a shift of the key.  From a sample T lies up to a fraction of an octave
// above key_lo: the window is one octave (2^23 keys).  After a warm start key_lo is kWarmBelow keys (1/8 octave,
// 8.3 %) below the previous T and the window half an octave, so a threshold between 0.92 and 1.3 times the
// previous one is found by the first pass: narrower bins, fewer entries to rank.  A candidate costs little (an
// 8-byte store), a failed guess a second pass over the row, hence the generous margin.
constexpr uint32_t kShiftCold = 11, kShiftWarm = 10;
constexpr uint32_t kWarmBelow = 1u << 20;
constexpr int kTieCap = 1024;                // entries of T's bin that are ranked directly (one per thread)
constexpr int kWarmSlots = 1;                // remembered thresholds per row (TopkArgs::warm = 1 .. kWarmSlots)
enum CollectMode { kColdPass = 0, kWarmPass = 1, kSecondPass = 2 };

struct __attribute__((aligned(64))) RowInfo {     // one cache line per row
    uint32_t key_lo, shift;       // lower bound of the candidate keys and bin width (first collect pass)
    uint32_t key_lo2, shift2;     // ... of the second pass, valid if use2
    uint32_t use2;                // the second pass redid this row: its histogram is hist_b
    uint32_t warm_used;           // the first pass started from a remembered threshold
    uint32_t failed;              // kRowFailed: the row went to the exact one-workgroup algorithm in the count kernel;
                                  // kRowCrowded: T's bin holds more than kTieCap candidates (see tie_min, tie_max)
    uint32_t bin_a, need_a;       // bin of T; entries still needed from that bin
    uint32_t ntie;                // length of the tie list
    uint32_t M;                   // candidates of the first pass (zero between calls)
    uint32_t q;                   // number of entries equal to the threshold key T that are kept
    uint32_t warm_T[kWarmSlots], warm_ok[kWarmSlots];   // thresholds T of earlier calls (the last call's: warm_T[0] if warm == 0)
    uint32_t tie_min, tie_max;    // crowded bin: smallest and largest key in it.  Equal: T is that key (many equal
                                  // magnitudes at the threshold, e.g. zeros), no ranking needed.  Different: the
                                  // exact one-workgroup algorithm, in the emit kernel.
};
enum { kRowFine = 0, kRowFailed = 1, kRowCrowded = 2 };
static_assert(sizeof(RowInfo) == 64, "one cache line");

struct Ws {
    uint32_t *hist_a, *hist_b;            // [n][kHistBins] each, kept zero between calls
    RowInfo *info;                        // [n]
    uint32_t *slot_cnt, *slot_above;      // [n][nslot] candidates of a slot; those in bins above T's
    uint32_t *slot_inbin;                 // [n][nslot] those in T's bin (written for crowded bins only)
    uint2 *tie;                           // [n][kTieCap] (position, key) of the candidates in T's bin
    uint2 *cand;                          // [n][nslot][L] (position, value bits) of the candidates
    int64_t L;                            // entries per wavefront piece = slot capacity
    int64_t nslot;                        // pieces per row
    int64_t G;                            // collect workgroups per row
};

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

void plan(int32_t n, int64_t d, Ws *w) {
    // one 1024-thread workgroup per CU; two for inputs of 2^26 entries and more (the collect kernels need 44
    // registers per lane and 36 KB of LDS, so two are resident).  Measured: short inputs lose with a second
    // workgroup per CU (each repeats the sampling prologue), long ones with fewer or more than two.
    int64_t max_g = ((int64_t)n * d >= ((int64_t)1 << 26) ? 512 : 256) / n;
    if (max_g < 1) max_g = 1;
    if (max_g > kMaxSlots / kBlkWaves) max_g = kMaxSlots / kBlkWaves;
    int64_t g = (d + kBlkWaves * 2048 - 1) / (kBlkWaves * 2048);   // at least 2048 entries per piece
    if (g > max_g) g = max_g;
    if (g < 1) g = 1;
    const int64_t pieces = g * kBlkWaves;
    int64_t L = (d + pieces - 1) / pieces;
    L = (L + 2047) / 2048 * 2048;            // whole load groups (4 steps of 64 lanes x 4 entries), and whole
                                             // blocks of the aggregation's message index (256 or 2048 coordinates)
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
    // the leading part (histograms, row records) starts at zero: launch_topk_split_reset
    char *ha = take(sizeof(uint32_t) * (size_t)n * kHistBins);
    char *hb = take(sizeof(uint32_t) * (size_t)n * kHistBins);
    char *inf = take(sizeof(RowInfo) * (size_t)n);
    const size_t slots = sizeof(uint32_t) * (size_t)n * tmp.nslot;
    char *s0 = take(slots), *s1 = take(slots), *s2 = take(slots);
    char *tl = take(sizeof(uint2) * (size_t)n * kTieCap);
    char *cd = take(sizeof(uint2) * (size_t)n * tmp.nslot * tmp.L);
    if (w) {
        *w = tmp;
        w->hist_a = (uint32_t *)ha; w->hist_b = (uint32_t *)hb;
        w->info = (RowInfo *)inf;
        w->slot_cnt = (uint32_t *)s0; w->slot_above = (uint32_t *)s1; w->slot_inbin = (uint32_t *)s2;
        w->tie = (uint2 *)tl;
        w->cand = (uint2 *)cd;
    }
    return off;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Bin of a candidate key (key >= key_lo) in the candidates' histogram.
__device__ __forceinline__ uint32_t bin_of(uint32_t key, uint32_t key_lo, uint32_t shift) {
    const uint32_t b = (key - key_lo) >> shift;
    return b < (uint32_t)kHistBins - 1u ? b : (uint32_t)kHistBins - 1u;
}

// exclusive prefix sum over the workgroup's threads; total returned through *total
template <int THREADS>
__device__ uint32_t cand_block_scan(uint32_t v, uint32_t *lds_wave /*[THREADS / 64]*/, uint32_t *total) {
    const uint32_t incl = wave_inclusive_scan(v);
    const int wave = threadIdx.x / kWave;
    __syncthreads();                       // lds_wave may still be in use by a previous scan
    if (lane_id() == kWave - 1) lds_wave[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (int v2 = 0; v2 < THREADS / kWave; ++v2) {
        const uint32_t t = lds_wave[v2];
        if (v2 < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

__device__ void zero_global_hist(uint32_t *hist, int bins) {
    for (int i = threadIdx.x; i < bins; i += blockDim.x) hist[i] = 0u;
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

// Lower bound of the candidate keys from the sample, identical in every workgroup of a row (it depends on
// the data only): the lower edge of the bin, in a histogram of the keys' 12 leading bits (1/16 octave), that holds
// the sample's r-th largest key.  A finer bound would save a few per cent of the candidates, which cost little,
// for a second histogram pass, which costs a microsecond in every workgroup.  0 means "every entry is a candidate".
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
    const uint32_t key_lo = s.bin << (kBits2 + kBits3);
    __syncthreads();
    return key_lo;
}

// Per-wavefront staging ring in LDS: candidates (position, value bits) are appended here and leave for the slot
// in global memory 64 at a time, as one full-width 8-byte store, instead of as many scattered stores.
constexpr uint32_t kRing = 128;              // entries of a staging ring (power of two, >= 128)
struct StageRing {
    uint2 e[kRing];
};

// What a wavefront needs to classify and count candidates.
struct CandFilter {
    uint32_t key_lo, shift;
    uint32_t *hist;          // the workgroup's LDS histogram
};

// Writes the entries [flushed, flushed + count) of the ring (count <= 64) to the slot and counts them into the
// histogram (here, with all lanes busy, rather than where they are found, a few lanes at a time).
__device__ __forceinline__ void ring_to_slot(const StageRing &ring, uint32_t flushed, uint32_t count, int lane,
                                             uint2 *slot, const CandFilter &f) {
    if ((uint32_t)lane < count) {
        const uint2 rec = ring.e[(flushed + lane) & (kRing - 1)];
        slot[flushed + lane] = rec;
        atomicAdd(&f.hist[bin_of(rec.y & 0x7fffffffu, f.key_lo, f.shift)], 1u);
    }
}

// Appends the candidates among one step's entries (VEC per lane, lane-major order) to the slot.
// FULL: every entry of the step lies inside the piece, no bounds checks.
// cnt = candidates so far, flushed = how many of them are already in global memory (cnt - flushed < 64
// between calls; both are uniform over the wavefront).
template <int VEC, bool FULL>
__device__ __forceinline__ void append_candidates(const float (&v)[VEC], int64_t e0, int64_t hi, const CandFilter &f,
                                                  StageRing &ring, int lane, uint2 *slot, uint32_t &cnt,
                                                  uint32_t &flushed) {
    bool c[VEC];
    uint32_t below = 0, all = 0;
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        c[t] = (FULL || e0 + t < hi) && mag_key(v[t]) >= f.key_lo;
        const uint64_t m = __ballot(c[t]);
        below += lanes_below(m);
        all += popc64(m);
    }
    if (all == 0) return;
    uint32_t pos = cnt + below;
    if (all > 64) {        // a dense step would not fit the ring: drain it, then store directly
        ring_to_slot(ring, flushed, cnt - flushed, lane, slot, f);
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            if (c[t]) {
                slot[pos] = make_uint2((uint32_t)(e0 + t), __float_as_uint(v[t]));
                atomicAdd(&f.hist[bin_of(mag_key(v[t]), f.key_lo, f.shift)], 1u);
                ++pos;
            }
        }
        cnt += all;
        flushed = cnt;
        return;
    }
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        if (c[t]) {
            ring.e[pos & (kRing - 1)] = make_uint2((uint32_t)(e0 + t), __float_as_uint(v[t]));
            ++pos;
        }
    }
    cnt += all;
    if (cnt - flushed > kRing - 64) {        // keep room for the next step's candidates (at most 64)
        __builtin_amdgcn_wave_barrier();
        ring_to_slot(ring, flushed, 64, lane, slot, f);
        flushed += 64;
    }
}

// Writes what is left in the ring at the end of a piece.
__device__ __forceinline__ void drain_ring(const StageRing &ring, uint32_t flushed, uint32_t cnt, int lane,
                                           uint2 *slot, const CandFilter &f) {
    __builtin_amdgcn_wave_barrier();
    for (; flushed < cnt; flushed += 64)
        ring_to_slot(ring, flushed, cnt - flushed < 64 ? cnt - flushed : 64, lane, slot, f);
}

// A wavefront walks its piece in steps of 64*VEC entries (VEC = 4 needs 16-byte aligned rows), U steps per
// group (VEC = 1: four).  Whole groups are loaded without any bounds check so that all loads of a group
// are in flight together; only the last piece of a row has a checked tail.
// MODE: kColdPass key_lo from the sample; kWarmPass from the threshold remembered in slot p.warm if there is
// one, else from the sample; kSecondPass: only rows whose warm start failed, from the sample, into hist_b.
template <int VEC, bool DIFF, int MODE, int U>
__global__ __launch_bounds__(kBlk) void split_collect_kernel(TopkArgs p, Ws w) {
    __shared__ RowShared s;
    __shared__ StageRing rings[kBlkWaves];
    __shared__ uint32_t wg_total;
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    RowInfo *info = w.info + row;
    CandFilter f;
    f.shift = kShiftCold;
    f.hist = s.hist;
    uint32_t *merged = w.hist_a + row * kHistBins;
    uint32_t *row_total = &info->M;
    if constexpr (MODE == kSecondPass) {
        // The guess of the first pass held if it kept at least k candidates and the k-th largest of them lies
        // inside the histogram's window, i.e. fewer than k fell into the last bin: then this pass ends here.
        const uint32_t warm_used = info->warm_used, M = info->M, beyond = merged[kHistBins - 1];
        if (!warm_used) return;                      // a cold first pass: what fails goes to the exact algorithm
        if (M >= (uint32_t)p.k && beyond < (uint32_t)p.k) return;
        f.key_lo = estimate_key_lo<DIFF>(s, a, b, d, p.k);
        merged = w.hist_b + row * kHistBins;
        row_total = nullptr;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            info->key_lo2 = f.key_lo;
            info->shift2 = f.shift;
            info->use2 = 1u;
        }
    } else {
        bool warm = false;
        if constexpr (MODE == kWarmPass) warm = info->warm_ok[p.warm - 1] != 0u;
        if (warm) {
            const uint32_t T = info->warm_T[p.warm - 1];
            f.key_lo = T > kWarmBelow ? T - kWarmBelow : 0u;
            f.shift = kShiftWarm;
        } else {
            f.key_lo = estimate_key_lo<DIFF>(s, a, b, d, p.k);
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            info->key_lo = f.key_lo;
            info->shift = f.shift;
            info->use2 = 0u;
            info->ntie = 0u;                 // the count kernel appends to the list
            info->tie_min = 0xffffffffu;
            info->tie_max = 0u;
            info->warm_used = warm ? 1u : 0u;
        }
    }
    for (int i = threadIdx.x; i < kHistBins; i += kBlk) s.hist[i] = 0u;
    if (threadIdx.x == 0) wg_total = 0u;
    __syncthreads();

    const int wave = threadIdx.x / kWave, lane = lane_id();
    // the first pass has a wavefront per slot; the second pass, which seldom has work, runs on a small grid
    for (int64_t slot_no = (int64_t)blockIdx.x * kBlkWaves + wave; slot_no < w.nslot;
         slot_no += (int64_t)gridDim.x * kBlkWaves) {
        StageRing &ring = rings[wave];
        const int64_t lo = slot_no * w.L;
        const int64_t hi = lo + w.L < d ? lo + w.L : d;
        uint2 *slot = w.cand + (row * w.nslot + slot_no) * w.L;
        uint32_t cnt = 0, flushed = 0;
        constexpr int kStep = kWave * VEC, kUnroll = VEC == 4 ? U : 4, kGroup = kStep * kUnroll;
        int64_t base = lo;
        if constexpr (VEC == 4) {
            // Groups of U steps, two register buffers: the next group's loads are issued before this group is
            // filtered, so that a wavefront has loads in flight while it computes.  After the last group the
            // "next" loads all read the piece's first 16 bytes (one cached line) instead of sitting behind a
            // branch.  What is in flight per compute unit is 1024 lanes x workgroups per unit x arrays x 2 U x 16
            // bytes; measured best at 64 to 128 KB (see launch_collect).
            float4 va[kUnroll], vb[kUnroll];
            if (base + kGroup <= hi) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = stream_load4(a + base + u * kStep + lane * 4);
                    if constexpr (DIFF) vb[u] = stream_load4(b + base + u * kStep + lane * 4);
                }
            }
            for (; base + kGroup <= hi; base += kGroup) {
                const bool more = base + 2 * kGroup <= hi;
                float4 na[kUnroll], nb[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int64_t at = more ? base + kGroup + u * kStep + lane * 4 : lo;
                    na[u] = stream_load4(a + at);
                    if constexpr (DIFF) nb[u] = stream_load4(b + at);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    float v[VEC] = {va[u].x, va[u].y, va[u].z, va[u].w};
                    if constexpr (DIFF) {
                        v[0] -= vb[u].x; v[1] -= vb[u].y; v[2] -= vb[u].z; v[3] -= vb[u].w;
                    }
                    append_candidates<VEC, true>(v, base + u * kStep + lane * VEC, hi, f, ring, lane, slot, cnt, flushed);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = na[u];
                    if constexpr (DIFF) vb[u] = nb[u];
                }
            }
        } else {
            for (; base + kGroup <= hi; base += kGroup) {
                float v[kUnroll][VEC];
                float vb[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    v[u][0] = stream_load(a + base + u * kStep + lane);
                    if constexpr (DIFF) vb[u] = stream_load(b + base + u * kStep + lane);
                }
                if constexpr (DIFF) {
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) v[u][0] -= vb[u];
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    append_candidates<VEC, true>(v[u], base + u * kStep + lane * VEC, hi, f, ring, lane, slot, cnt, flushed);
            }
        }
        for (; base < hi; base += kStep) {           // checked tail, entry by entry
            const int64_t e0 = base + lane * VEC;
            float v[VEC];
#pragma unroll
            for (int t = 0; t < VEC; ++t) v[t] = e0 + t < hi ? load_v<DIFF>(a, b, e0 + t) : 0.f;
            append_candidates<VEC, false>(v, e0, hi, f, ring, lane, slot, cnt, flushed);
        }
        drain_ring(ring, flushed, cnt, lane, slot, f);
        if (lane == 0) {
            w.slot_cnt[row * w.nslot + slot_no] = cnt;
            atomicAdd(&wg_total, cnt);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHistBins; i += kBlk) {
        const uint32_t c = s.hist[i];
        if (c) atomicAdd(merged + i, c);
    }
    if (row_total && threadIdx.x == 0 && wg_total) atomicAdd(row_total, wg_total);
}

// ---------------------------------------------------------------- collect, two selections in one pass
// Algorithm 3 (EF21+) selects from two vectors built of the same arrays: the gradient s itself (line 5) and the
// difference s - g_i (line 6), and needs the squared norms of both (line 7).  This kernel reads s and g_i once
// and does the work of two collect passes and of the norm pass: candidates, histograms and slot counts of the
// difference go to workspace `wm` (arguments pm: a = s, b = g_i), those of s to workspace `wp` (warm-start memory
// warm_p), and every wavefront leaves (sum s^2, sum (s - g_i)^2) over its piece in norms[row][slot], the
// differences of the stored values taken exactly in fp64 and the sums in a fixed order.
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

template <int VEC, bool WARM, int U>
__global__ __launch_bounds__(kBlk) void split_collect_pair_kernel(TopkArgs pm, Ws wm, int warm_p, Ws wp,
                                                                  double2 *__restrict__ norms) {
    __shared__ RowShared s;                      // its histogram serves the sampling, then the difference
    __shared__ uint32_t hist_p[kHistBins];
    __shared__ StageRing rings_m[kBlkWaves], rings_p[kBlkWaves];
    __shared__ uint32_t wg_total_m, wg_total_p;
    const int64_t row = blockIdx.y, d = pm.d;
    const float *a = pm.a + row * d, *b = pm.b + row * d;
    RowInfo *info_m = wm.info + row, *info_p = wp.info + row;
    CandFilter fm, fp;
    fm.hist = s.hist;
    fp.hist = hist_p;
    const bool warm_m = WARM && info_m->warm_ok[pm.warm - 1] != 0u, warm_pl = WARM && info_p->warm_ok[warm_p - 1] != 0u;
    if (warm_m) {
        const uint32_t T = info_m->warm_T[pm.warm - 1];
        fm.key_lo = T > kWarmBelow ? T - kWarmBelow : 0u;
        fm.shift = kShiftWarm;
    } else {
        fm.key_lo = estimate_key_lo<true>(s, a, b, d, pm.k);
        fm.shift = kShiftCold;
    }
    if (warm_pl) {
        const uint32_t T = info_p->warm_T[warm_p - 1];
        fp.key_lo = T > kWarmBelow ? T - kWarmBelow : 0u;
        fp.shift = kShiftWarm;
    } else {
        fp.key_lo = estimate_key_lo<false>(s, a, nullptr, d, pm.k);
        fp.shift = kShiftCold;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        info_m->key_lo = fm.key_lo; info_m->shift = fm.shift; info_m->use2 = 0u; info_m->ntie = 0u;
        info_m->tie_min = 0xffffffffu; info_m->tie_max = 0u;
        info_m->warm_used = warm_m ? 1u : 0u;
        info_p->key_lo = fp.key_lo; info_p->shift = fp.shift; info_p->use2 = 0u; info_p->ntie = 0u;
        info_p->tie_min = 0xffffffffu; info_p->tie_max = 0u;
        info_p->warm_used = warm_pl ? 1u : 0u;
    }
    for (int i = threadIdx.x; i < kHistBins; i += kBlk) {
        s.hist[i] = 0u;
        hist_p[i] = 0u;
    }
    if (threadIdx.x == 0) {
        wg_total_m = 0u;
        wg_total_p = 0u;
    }
    __syncthreads();

    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t slot_no = (int64_t)blockIdx.x * kBlkWaves + wave;
    if (slot_no < wm.nslot) {
        StageRing &ring_m = rings_m[wave], &ring_p = rings_p[wave];
        const int64_t lo = slot_no * wm.L;
        const int64_t hi = lo + wm.L < d ? lo + wm.L : d;
        uint2 *slot_m = wm.cand + (row * wm.nslot + slot_no) * wm.L;
        uint2 *slot_p = wp.cand + (row * wp.nslot + slot_no) * wp.L;
        uint32_t cnt_m = 0, flushed_m = 0, cnt_p = 0, flushed_p = 0;
        double sq_s = 0.0, sq_v = 0.0;
        constexpr int kStep = kWave * VEC, kUnroll = VEC == 4 ? U : 4, kGroup = kStep * kUnroll;
        int64_t base = lo;
        // one group: the squared norms of line 7, the difference of line 6, both filters
        auto filter_group = [&](float (&vs)[kUnroll][VEC], float (&vd)[kUnroll][VEC]) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
                for (int t = 0; t < VEC; ++t) {
                    const double sv = (double)vs[u][t], dv = sv - (double)vd[u][t];      // exact
                    sq_s += sv * sv;
                    sq_v += dv * dv;
                    vd[u][t] = vs[u][t] - vd[u][t];                                      // line 6: one fp32 subtraction
                }
                const int64_t e0 = base + u * kStep + lane * VEC;
                append_candidates<VEC, true>(vs[u], e0, hi, fp, ring_p, lane, slot_p, cnt_p, flushed_p);
                append_candidates<VEC, true>(vd[u], e0, hi, fm, ring_m, lane, slot_m, cnt_m, flushed_m);
            }
        };
        if constexpr (VEC == 4) {
            // two register buffers, as in split_collect_kernel: the next group's loads before this group's work
            float4 va[kUnroll], vb[kUnroll];
            if (base + kGroup <= hi) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = stream_load4(a + base + u * kStep + lane * 4);
                    vb[u] = stream_load4(b + base + u * kStep + lane * 4);
                }
            }
            for (; base + kGroup <= hi; base += kGroup) {
                const bool more = base + 2 * kGroup <= hi;
                float4 na[kUnroll], nb[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int64_t at = more ? base + kGroup + u * kStep + lane * 4 : lo;
                    na[u] = stream_load4(a + at);
                    nb[u] = stream_load4(b + at);
                }
                float vs[kUnroll][VEC], vd[kUnroll][VEC];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    vs[u][0] = va[u].x; vs[u][1] = va[u].y; vs[u][2] = va[u].z; vs[u][3] = va[u].w;
                    vd[u][0] = vb[u].x; vd[u][1] = vb[u].y; vd[u][2] = vb[u].z; vd[u][3] = vb[u].w;
                }
                filter_group(vs, vd);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = na[u];
                    vb[u] = nb[u];
                }
            }
        } else {
            for (; base + kGroup <= hi; base += kGroup) {
                float vs[kUnroll][VEC], vd[kUnroll][VEC];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    vs[u][0] = stream_load(a + base + u * kStep + lane);
                    vd[u][0] = stream_load(b + base + u * kStep + lane);
                }
                filter_group(vs, vd);
            }
        }
        for (; base < hi; base += kStep) {           // checked tail, entry by entry
            const int64_t e0 = base + lane * VEC;
            float vs[VEC], vd[VEC];
#pragma unroll
            for (int t = 0; t < VEC; ++t) {
                const bool in = e0 + t < hi;
                const float sv = in ? a[e0 + t] : 0.f, bv = in ? b[e0 + t] : 0.f;
                const double dv = (double)sv - (double)bv;
                sq_s += (double)sv * (double)sv;
                sq_v += dv * dv;
                vs[t] = sv;
                vd[t] = sv - bv;
            }
            append_candidates<VEC, false>(vs, e0, hi, fp, ring_p, lane, slot_p, cnt_p, flushed_p);
            append_candidates<VEC, false>(vd, e0, hi, fm, ring_m, lane, slot_m, cnt_m, flushed_m);
        }
        drain_ring(ring_p, flushed_p, cnt_p, lane, slot_p, fp);
        drain_ring(ring_m, flushed_m, cnt_m, lane, slot_m, fm);
        sq_s = wave_sum_f64(sq_s);
        sq_v = wave_sum_f64(sq_v);
        if (lane == 0) {
            wm.slot_cnt[row * wm.nslot + slot_no] = cnt_m;
            wp.slot_cnt[row * wp.nslot + slot_no] = cnt_p;
            atomicAdd(&wg_total_m, cnt_m);
            atomicAdd(&wg_total_p, cnt_p);
            norms[row * wm.nslot + slot_no] = make_double2(sq_s, sq_v);
        }
    }
    __syncthreads();
    uint32_t *merged_m = wm.hist_a + row * kHistBins, *merged_p = wp.hist_a + row * kHistBins;
    for (int i = threadIdx.x; i < kHistBins; i += kBlk) {
        const uint32_t cm = s.hist[i], cp = hist_p[i];
        if (cm) atomicAdd(merged_m + i, cm);
        if (cp) atomicAdd(merged_p + i, cp);
    }
    if (threadIdx.x == 0) {
        if (wg_total_m) atomicAdd(&info_m->M, wg_total_m);
        if (wg_total_p) atomicAdd(&info_p->M, wg_total_p);
    }
}

// ---------------------------------------------------------------- count
// The exact one-workgroup algorithm on the original data for a row whose guess failed, and the message index of
// the row if the caller asked for one.  All kCandThreads threads of the workgroup must call.
template <bool DIFF, bool UPDATE>
__device__ void rescue_row(RowShared &rs, const TopkArgs &p, int64_t row) {
    row_topk<DIFF, UPDATE>(rs, p, row);
    if (p.agg_start) {                  // from the pairs just written
        __syncthreads();
        const int32_t *out = p.out_idx + row * p.k;
        int32_t *start = p.agg_start + row * (p.agg_nblk + 1);
        for (int64_t at = threadIdx.x; at < p.k; at += kCandThreads) {
            const int64_t b_cur = out[at] >> p.agg_shift;
            const int64_t b_prev = at > 0 ? out[at - 1] >> p.agg_shift : -1;
            for (int64_t b = b_prev + 1; b <= b_cur; ++b) start[b] = (int32_t)at;
            if (at == p.k - 1)
                for (int64_t b = b_cur + 1; b <= p.agg_nblk; ++b) start[b] = (int32_t)p.k;
        }
    }
}

// A wavefront of the count and emit kernels takes kSPW consecutive slots (one, or two where one would put more
// than a workgroup on every compute unit).  The first kPre steps of 64 candidates
// of each (clamped to the slot's capacity, a multiple of 1024) are loaded at the very start of the kernel, together
// with everything else whose address does not depend on the prologue, so that a workgroup waits for memory once,
// not once per step of its prologue.
constexpr int kPre = 4;

// Grid (slot blocks + 1, n).  Prologue of every workgroup: T's bin from the row's histogram, and whether the row
// failed (see the head of the file).  The last workgroup of a row is the rescue: it selects a failed row by the
// exact one-workgroup algorithm on the original data (DIFF and UPDATE matter here only).  The others: a slot's
// candidates in bins above T's are counted, those in T's bin go to the tie list.
template <bool DIFF, bool UPDATE, int kSPW>
__global__ __launch_bounds__(kCandThreads) void cand_count_kernel(TopkArgs p, Ws w) {
    constexpr int kWgSlots = kCandWaves * kSPW;      // slots per workgroup
    __shared__ RowShared rs;
    __shared__ uint32_t lds_wave[kCandWaves], lds_out[4];
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    const bool rescue = blockIdx.x == gridDim.x - 1;
    const int64_t sl_first = rescue ? 0 : (int64_t)blockIdx.x * kWgSlots + wave * kSPW;
    // everything whose address is known now
    const RowInfo ri = *info;
    constexpr int PER = kHistBins / kCandThreads;
    uint32_t h[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) h[j] = w.hist_a[row * kHistBins + kHistBins - 1 - (tid * PER + j)];
    uint32_t cnt[kSPW];
    const uint2 *slot[kSPW];
    uint2 c[kSPW][kPre];
#pragma unroll
    for (int s = 0; s < kSPW; ++s) {
        const bool active = !rescue && sl_first + s < w.nslot;
        const int64_t slc = active ? sl_first + s : 0;
        cnt[s] = w.slot_cnt[row * w.nslot + slc];
        slot[s] = w.cand + (row * w.nslot + slc) * w.L;
#pragma unroll
        for (int q = 0; q < kPre; ++q) c[s][q] = slot[s][q * kWave + lane];
        if (!active) cnt[s] = 0u;
    }

    const bool second = ri.use2 != 0u;
    const uint32_t key_lo = second ? ri.key_lo2 : ri.key_lo, shift = second ? ri.shift2 : ri.shift;
    if (second) {
#pragma unroll
        for (int j = 0; j < PER; ++j) h[j] = w.hist_b[row * kHistBins + kHistBins - 1 - (tid * PER + j)];
    }
    // T's bin: the largest bin b with count(bins > b) < k <= count(bins >= b)
    uint32_t mine = 0, total;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += h[j];
    const uint32_t higher = cand_block_scan<kCandThreads>(mine, lds_wave, &total);
    const uint32_t need = (uint32_t)p.k;
    if (higher < need && need <= higher + mine) {         // exactly one thread, if total >= k
        uint32_t run = higher;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (need > run && need <= run + h[j]) {
                lds_out[0] = (uint32_t)(kHistBins - 1 - (tid * PER + j));
                lds_out[1] = need - run;
                lds_out[2] = h[j];
            }
            run += h[j];
        }
    }
    __syncthreads();
    bool failed = total < need, crowded = false;                       // fewer than k candidates
    uint32_t bin_a = 0, need_a = 0;
    if (!failed) {
        bin_a = lds_out[0];
        need_a = lds_out[1];
        failed = bin_a == (uint32_t)kHistBins - 1u;                    // beyond the window
        crowded = !failed && lds_out[2] > (uint32_t)kTieCap;           // too many to list: see RowInfo::tie_min
    }
    if (rescue) {
        if (failed) rescue_row<DIFF, UPDATE>(rs, p, row);
        return;
    }
    if (blockIdx.x == 0 && tid == 0) {
        info->failed = failed ? kRowFailed : (crowded ? kRowCrowded : kRowFine);
        info->bin_a = bin_a;
        info->need_a = need_a;
        info->M = 0u;                        // consumed by the second collect pass: zero for the next call
        if (failed && p.warm > 0) info->warm_ok[p.warm - 1] = 0u;
    }
    if (failed) return;
    uint2 *tie = w.tie + row * kTieCap;
    uint32_t key_min = 0xffffffffu, key_max = 0u;
#pragma unroll
    for (int s = 0; s < kSPW; ++s) {
        uint32_t above = 0, inbin = 0;
        for (uint32_t j0 = 0; j0 < cnt[s]; j0 += kWave * kPre) {
            if (j0 > 0) {
#pragma unroll
                for (int q = 0; q < kPre; ++q) {
                    const uint32_t j = j0 + q * kWave + lane;
                    c[s][q] = slot[s][j < cnt[s] ? j : 0u];       // clamped: no load behind a branch
                }
            }
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                const uint32_t j = j0 + q * kWave + lane;
                const uint32_t key = c[s][q].y & 0x7fffffffu;
                const uint32_t bin = bin_of(key < key_lo ? key_lo : key, key_lo, shift);
                above += popc64(__ballot(j < cnt[s] && bin > bin_a));
                const bool in_bin = j < cnt[s] && bin == bin_a;
                if (!crowded) {
                    const uint32_t at = wave_append(in_bin, &info->ntie);
                    if (in_bin && at < (uint32_t)kTieCap) tie[at] = make_uint2(c[s][q].x, key);
                } else {
                    inbin += popc64(__ballot(in_bin));
                    key_min = in_bin && key < key_min ? key : key_min;
                    key_max = in_bin && key > key_max ? key : key_max;
                }
            }
        }
        if (lane == 0 && sl_first + s < w.nslot) {
            w.slot_above[row * w.nslot + sl_first + s] = above;
            if (crowded) w.slot_inbin[row * w.nslot + sl_first + s] = inbin;
        }
    }
    if (crowded) {
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) {
            const uint32_t lo_o = __shfl_xor(key_min, o, kWave), hi_o = __shfl_xor(key_max, o, kWave);
            key_min = lo_o < key_min ? lo_o : key_min;
            key_max = hi_o > key_max ? hi_o : key_max;
        }
        if (lane == 0 && key_min <= key_max) {
            atomicMin(&info->tie_min, key_min);
            atomicMax(&info->tie_max, key_max);
        }
    }
}

// Ordered emission by one wavefront that walks candidates in position order, 64 at a time: the running output
// offset, the ties seen so far, and (if asked for) the aggregation's message index, start[b] = output position of
// the first kept entry at or beyond coordinate b << shift.  A wavefront's span [span_lo, span_end) is a whole number
// of index blocks, so every block begins inside exactly one wavefront's span, and that wavefront writes its start:
// when it keeps the first entry at or beyond the block's first coordinate, or at the end of its span for the
// blocks that follow its last kept entry (all of them if it kept nothing).
template <bool DIFF, bool UPDATE>
struct Emitter {
    const TopkArgs &p;
    int64_t row;
    uint32_t T, q;               // threshold key; entries equal to T that are kept (the first q in position order)
    uint32_t out_run, eq_run;    // kept entries, and entries equal to T, before the next step
    int32_t *out_idx;
    float *out_val;
    int32_t *agg_start;
    int64_t last_b;              // index blocks up to here have their start
    int lane;

    __device__ Emitter(const TopkArgs &p_, int64_t row_, uint32_t T_, uint32_t q_, uint32_t gt_before,
                       uint32_t eq_before, int64_t span_lo, int lane_)
        : p(p_), row(row_), T(T_), q(q_), out_run(gt_before + (eq_before < q_ ? eq_before : q_)), eq_run(eq_before),
          out_idx(p_.out_idx + row_ * p_.k), out_val(p_.out_val + row_ * p_.k),
          agg_start(p_.agg_start ? p_.agg_start + row_ * (p_.agg_nblk + 1) : nullptr),
          last_b((span_lo >> p_.agg_shift) - 1), lane(lane_) {}

    // one step: `in` marks the lanes that hold a candidate (position rec.x, value bits rec.y); all lanes call.
    // have_b: b_pre is the value of b at the candidate's position, loaded by the caller beforehand.
    __device__ __forceinline__ void step(bool in, uint2 rec, bool have_b = false, float b_pre = 0.f) {
        const uint32_t key = rec.y & 0x7fffffffu;
        const bool gt = in && key > T, eq = in && key == T;
        const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
        const uint32_t eq_below = eq_run + lanes_below(m_eq);
        const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
        const bool keep = gt || (eq && eq_below < q);
        const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
        if (keep) {
            const float v = __uint_as_float(rec.y);
            out_idx[pos] = (int32_t)rec.x;
            out_val[pos] = v;
            if constexpr (UPDATE) {                      // Algorithm 2, line 6
                const int64_t at = row * p.d + (int64_t)rec.x;
                p.g_i[at] = (DIFF ? (have_b ? b_pre : p.b[at]) : 0.f) + v;
            }
        }
        if (agg_start) {
            const uint64_t m_keep = __ballot(keep);
            if (m_keep) {
                const int64_t b_cur = (int64_t)(rec.x >> p.agg_shift);
                const uint64_t lower = m_keep & ((1ull << lane) - 1ull);
                const int prev_lane = lower ? 63 - __clzll((long long)lower) : 0;
                const int64_t b_before = __shfl(b_cur, prev_lane, kWave);
                const int64_t b_prev = lower ? b_before : last_b;
                if (keep)
                    for (int64_t b = b_prev + 1; b <= b_cur; ++b) agg_start[b] = (int32_t)pos;
                last_b = __shfl(b_cur, 63 - __clzll((long long)m_keep), kWave);
            }
        }
        const uint32_t eq_next = eq_run + popc64(m_eq);
        out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_run < q ? eq_run : q));
        eq_run = eq_next;
    }

    // after the last step of a span that ends at span_end (clamped to the row's end by the caller)
    __device__ __forceinline__ void finish(int64_t span_end) {
        if (!agg_start) return;
        const int64_t b_last = ((span_end - 1) >> p.agg_shift) + (span_end == p.d ? 1 : 0);   // the row's end: start[nblk]
        for (int64_t b = last_b + 1 + lane; b <= b_last; b += kWave) agg_start[b] = (int32_t)out_run;
    }
};

// ---------------------------------------------------------------- emit
// Ordered emission.  Prologue of every workgroup: the tie list ranked (larger key first, lower position first
// among equal keys): the entry that need_a - 1 others precede is the last one kept, its key is T, and q counts it
// and the equal keys before it.  The output offset of a slot is the number of kept entries in all earlier slots:
// their candidates above T's bin (slot_above, summed by the workgroup) plus the listed entries before the slot's
// first position that are kept.  Grid (slot blocks + 1, n): the last workgroup of a row is a rescue, for a row
// whose crowded bin (see RowInfo::tie_min) turned out to hold different keys.  A crowded bin of equal keys needs no
// list: T is that key, and the ties before a slot are the earlier slots' entries of the bin (slot_inbin).
template <bool DIFF, bool UPDATE, int kSPW>
__global__ __launch_bounds__(kCandThreads) void cand_emit_kernel(TopkArgs p, Ws w) {
    constexpr int kWgSlots = kCandWaves * kSPW;      // slots per workgroup
    __shared__ RowShared rs;                     // the rescue's
    __shared__ uint32_t before_above[kCandWaves], own_above[kCandWaves], before_inbin[kCandWaves], own_inbin[kCandWaves];
    __shared__ uint32_t tie_key[kTieCap], tie_idx[kTieCap];
    __shared__ uint32_t sh_T, sh_q;
    static_assert(kTieCap <= kCandThreads, "one listed entry per thread");
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    const bool rescue = blockIdx.x == gridDim.x - 1;
    const int64_t sl0 = rescue ? 0 : (int64_t)blockIdx.x * kWgSlots, sl_first = sl0 + wave * kSPW;
    // everything whose address is known now
    const RowInfo ri = *info;
    const bool crowded = ri.failed == kRowCrowded;
    if (rescue) {
        if (crowded && ri.tie_min != ri.tie_max) rescue_row<DIFF, UPDATE>(rs, p, row);
        return;
    }
    const uint2 listed = w.tie[row * kTieCap + (tid < kTieCap ? tid : 0)];
    const uint32_t *slot_above = w.slot_above + row * w.nslot;
    const uint32_t *slot_inbin = w.slot_inbin + row * w.nslot;
    uint32_t part = 0, part_in = 0;
    for (int64_t t = tid; t < sl0; t += kCandThreads) {
        part += slot_above[t];
        if (crowded) part_in += slot_inbin[t];
    }
    uint32_t mine = 0, mine_in = 0, cnt[kSPW];
    const uint2 *slot[kSPW];
    uint2 c[kSPW][kPre];
#pragma unroll
    for (int s = 0; s < kSPW; ++s) {
        const bool active = sl_first + s < w.nslot;
        const int64_t slc = active ? sl_first + s : 0;
        mine += active ? slot_above[slc] : 0u;
        mine_in += active && crowded ? slot_inbin[slc] : 0u;
        cnt[s] = w.slot_cnt[row * w.nslot + slc];
        slot[s] = w.cand + (row * w.nslot + slc) * w.L;
#pragma unroll
        for (int q = 0; q < kPre; ++q) c[s][q] = slot[s][q * kWave + lane];
        if (!active) cnt[s] = 0u;
    }
    // Line 6 needs g_i at the kept positions, scattered over the row: the loads for the wavefront's first
    // candidates that can be kept (those in T's bin or above: T itself is not known yet) are issued here, with
    // everything else, instead of one step at a time between the stores of the emission.
    float bpre[kSPW][kPre];
    if constexpr (DIFF && UPDATE) {
        const uint32_t key_lo = ri.use2 != 0u ? ri.key_lo2 : ri.key_lo, shift = ri.use2 != 0u ? ri.shift2 : ri.shift;
#pragma unroll
        for (int s = 0; s < kSPW; ++s)
#pragma unroll
            for (int q = 0; q < kPre; ++q) {
                const uint32_t key = c[s][q].y & 0x7fffffffu;
                const bool have = (uint32_t)(q * kWave + lane) < cnt[s] &&
                                  bin_of(key < key_lo ? key_lo : key, key_lo, shift) >= ri.bin_a;
                bpre[s][q] = p.b[row * p.d + (have ? (int64_t)c[s][q].x : 0)];
            }
    }

    if (blockIdx.x == 0) {                       // the histograms are consumed: zero for the next call
        zero_global_hist(w.hist_a + row * kHistBins, kHistBins);
        if (ri.use2 != 0u) zero_global_hist(w.hist_b + row * kHistBins, kHistBins);
    }
    if (ri.failed == kRowFailed || (crowded && ri.tie_min != ri.tie_max)) return;     // the whole workgroup
    const uint32_t ntie = crowded ? 0u : (ri.ntie < (uint32_t)kTieCap ? ri.ntie : (uint32_t)kTieCap);
    const uint32_t my_idx = listed.x, my_key = listed.y;
    if ((uint32_t)tid < ntie) {
        tie_idx[tid] = my_idx;
        tie_key[tid] = my_key;
    }
    __syncthreads();
    if ((uint32_t)tid < ntie) {
        uint32_t larger = 0, equal_before = 0;
        for (uint32_t j = 0; j < ntie; ++j) {
            const uint32_t kj = tie_key[j], ij = tie_idx[j];
            larger += kj > my_key ? 1u : 0u;
            equal_before += (kj == my_key && ij < my_idx) ? 1u : 0u;
        }
        if (larger + equal_before == ri.need_a - 1u) {       // exactly one thread
            sh_T = my_key;
            sh_q = equal_before + 1u;
        }
    }
    __syncthreads();
    const uint32_t T = crowded ? ri.tie_min : sh_T, q = crowded ? ri.need_a : sh_q;
    if (blockIdx.x == 0 && tid == 0) {
        info->q = q;
        const int mem = p.warm > 0 ? p.warm - 1 : 0;
        info->warm_T[mem] = T;
        info->warm_ok[mem] = p.warm > 0 ? 1u : 0u;
    }

    part = wave_sum_u32(part);
    part_in = wave_sum_u32(part_in);
    // listed entries before this wavefront's first position: kept ones above T, and ties
    const uint32_t my_lo = (uint32_t)(sl_first * w.L);
    uint32_t list_gt = 0, list_eq = 0;
    for (uint32_t j = lane; j < ntie; j += kWave) {
        const uint32_t kj = tie_key[j];
        if (tie_idx[j] < my_lo) {
            list_gt += kj > T ? 1u : 0u;
            list_eq += kj == T ? 1u : 0u;
        }
    }
    list_gt = wave_sum_u32(list_gt);
    list_eq = wave_sum_u32(list_eq);
    if (lane == 0) {
        before_above[wave] = part;
        own_above[wave] = mine;
        before_inbin[wave] = part_in;
        own_inbin[wave] = mine_in;
    }
    __syncthreads();
    if (sl_first >= w.nslot) return;
    uint32_t gt_run = list_gt, eq_run = list_eq;
    for (int v = 0; v < kCandWaves; ++v) {
        gt_run += before_above[v] + (v < wave ? own_above[v] : 0u);
        eq_run += before_inbin[v] + (v < wave ? own_inbin[v] : 0u);      // zero unless the bin is crowded
    }
    Emitter<DIFF, UPDATE> em(p, row, T, q, gt_run, eq_run, sl_first * w.L, lane);
#pragma unroll
    for (int s = 0; s < kSPW; ++s) {             // consecutive slots: the running offsets carry over
        for (uint32_t j0 = 0; j0 < cnt[s]; j0 += kWave * kPre) {
            if (j0 > 0) {
#pragma unroll
                for (int u = 0; u < kPre; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    c[s][u] = slot[s][j < cnt[s] ? j : 0u];      // clamped: no load behind a branch
                }
            }
#pragma unroll
            for (int u = 0; u < kPre; ++u) {
                if constexpr (DIFF && UPDATE) em.step(j0 + u * kWave + lane < cnt[s], c[s][u], j0 == 0, bpre[s][u]);
                else em.step(j0 + u * kWave + lane < cnt[s], c[s][u]);
            }
        }
    }
    const int64_t span_end = (sl_first + kSPW) * w.L;
    em.finish(span_end < p.d ? span_end : p.d);
}

__global__ __launch_bounds__(kCandThreads) void zero_words_kernel(uint32_t *p, size_t words) {
    const size_t stride = (size_t)gridDim.x * kCandThreads;
    for (size_t i = (size_t)blockIdx.x * kCandThreads + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

template <int VEC, bool DIFF, int U>
void launch_collect_u(const TopkArgs &p, const Ws &w, int mode, const dim3 &grid, hipStream_t stream) {
    const dim3 block(kBlk);
    if (mode == kColdPass) hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF, kColdPass, U>), grid, block, 0, stream, p, w);
    else if (mode == kWarmPass) hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF, kWarmPass, U>), grid, block, 0, stream, p, w);
    else hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF, kSecondPass, U>), grid, block, 0, stream, p, w);
}

template <int VEC, bool DIFF>
void launch_collect(const TopkArgs &p, const Ws &w, int mode, hipStream_t stream) {
    // the second pass has work only after a failed guess: about 64 workgroups, which loop over the slots
    int64_t g = w.G;
    if (mode == kSecondPass) g = std::max<int64_t>(1, std::min<int64_t>(w.G, 64 / p.n));
    const dim3 grid((unsigned)g, (unsigned)p.n);
    // Steps per group.  Two arrays and two workgroups per compute unit: one step (128 KB in flight per unit; C4:
    // 138 us against 142 with two steps and 147 without the second buffer); otherwise two (one array, one workgroup
    // per unit, the C1 call: 31.7 us against 36 with one step and 33 with four).
    if constexpr (VEC == 4 && DIFF) {
        if (g * p.n > 256) {
            launch_collect_u<VEC, DIFF, 1>(p, w, mode, grid, stream);
            return;
        }
    }
    launch_collect_u<VEC, DIFF, 2>(p, w, mode, grid, stream);
}

void launch_collect_any(const TopkArgs &p, const Ws &w, int mode, hipStream_t stream) {
    const bool diff = p.b != nullptr;
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0) && (!diff || (uintptr_t)p.b % 16 == 0);
    if (vec4 && diff) launch_collect<4, true>(p, w, mode, stream);
    else if (vec4) launch_collect<4, false>(p, w, mode, stream);
    else if (diff) launch_collect<1, true>(p, w, mode, stream);
    else launch_collect<1, false>(p, w, mode, stream);
}

// ---------------------------------------------------------------- k = 1: the entry of largest magnitude
// Top-1 (the compressor of the paper's first experiment) needs no threshold and no candidates: every thread
// keeps the best entry of its share as one 64-bit word, key << 32 | ~position (a larger word = a larger
// magnitude, or the same magnitude at a lower position), the words are reduced over the wavefront and the
// workgroup, and one 64-bit atomic maximum per workgroup lands in the row's slot (the first two words of the
// row's histogram in the workspace, which are zero between calls).  A second, tiny kernel turns the slot into
// the message, applies line 6 and clears the slot.
constexpr int kArgThreads = 256, kArgWaves = kArgThreads / kWave;

template <int VEC, bool DIFF>
__global__ __launch_bounds__(kArgThreads) void argmax_stream_kernel(TopkArgs p, Ws w, int64_t piece) {
    __shared__ unsigned long long best_of_wave[kArgWaves];
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    const int64_t lo = (int64_t)blockIdx.x * piece, hi = lo + piece < d ? lo + piece : d;
    unsigned long long best = 0ull;
    auto see = [&](float v, int64_t e) {
        const unsigned long long word = ((unsigned long long)mag_key(v) << 32) | (0xffffffffu - (uint32_t)e);
        best = word > best ? word : best;
    };
    if constexpr (VEC == 4) {
        constexpr int kUnroll = DIFF ? 4 : 8;
        constexpr int64_t kStep = (int64_t)kArgThreads * 4;
        int64_t e = lo + (int64_t)threadIdx.x * 4;               // piece % 4 == 0: whole float4s inside [lo, hi)
        for (; e + (kUnroll - 1) * kStep + 4 <= hi; e += kUnroll * kStep) {
            float4 va[kUnroll], vb[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                va[u] = stream_load4(a + e + u * kStep);
                if constexpr (DIFF) vb[u] = stream_load4(b + e + u * kStep);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if constexpr (DIFF) {
                    va[u].x -= vb[u].x;
                    va[u].y -= vb[u].y;
                    va[u].z -= vb[u].z;
                    va[u].w -= vb[u].w;
                }
                const int64_t e0 = e + u * kStep;
                see(va[u].x, e0);
                see(va[u].y, e0 + 1);
                see(va[u].z, e0 + 2);
                see(va[u].w, e0 + 3);
            }
        }
        for (; e + 4 <= hi; e += kStep) {
            float4 va = stream_load4(a + e);
            if constexpr (DIFF) {
                const float4 vb = stream_load4(b + e);
                va.x -= vb.x;
                va.y -= vb.y;
                va.z -= vb.z;
                va.w -= vb.w;
            }
            see(va.x, e);
            see(va.y, e + 1);
            see(va.z, e + 2);
            see(va.w, e + 3);
        }
    } else {
        for (int64_t e = lo + threadIdx.x; e < hi; e += kArgThreads) see(load_v<DIFF>(a, b, e), e);
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const unsigned long long other = __shfl_xor(best, o, kWave);
        best = other > best ? other : best;
    }
    if (lane_id() == 0) best_of_wave[threadIdx.x / kWave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int v = 1; v < kArgWaves; ++v) best = best_of_wave[v] > best ? best_of_wave[v] : best;
        if (lo < hi) atomicMax(reinterpret_cast<unsigned long long *>(w.hist_a + row * kHistBins), best);
    }
}

template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kArgThreads) void argmax_finish_kernel(TopkArgs p, Ws w) {
    const int64_t row = (int64_t)blockIdx.x * kArgThreads + threadIdx.x;
    if (row >= p.n) return;
    unsigned long long *slot = reinterpret_cast<unsigned long long *>(w.hist_a + row * kHistBins);
    const int64_t e = (int64_t)(0xffffffffu - (uint32_t)(*slot & 0xffffffffull));
    *slot = 0ull;
    const float bv = DIFF ? p.b[row * p.d + e] : 0.f;
    const float v = DIFF ? p.a[row * p.d + e] - bv : p.a[row * p.d + e];
    p.out_idx[row] = (int32_t)e;                                // k == 1: one pair per row
    p.out_val[row] = v;
    if (UPDATE) p.g_i[row * p.d + e] = bv + v;                  // Algorithm 2, line 6
}

hipError_t launch_argmax(const TopkArgs &p, const Ws &w, hipStream_t stream, const Marker &mk) {
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0) && (!diff || (uintptr_t)p.b % 16 == 0);
    int64_t G = 1024 / p.n;                                     // about four workgroups of 256 per compute unit
    if (G < 1) G = 1;
    int64_t piece = (p.d + G - 1) / G;
    piece = (piece + 3) & ~(int64_t)3;
    if (piece < 4096) piece = 4096;
    G = (p.d + piece - 1) / piece;
    const dim3 grid((unsigned)G, (unsigned)p.n), block(kArgThreads);
    if (vec4 && diff) hipLaunchKernelGGL((argmax_stream_kernel<4, true>), grid, block, 0, stream, p, w, piece);
    else if (vec4) hipLaunchKernelGGL((argmax_stream_kernel<4, false>), grid, block, 0, stream, p, w, piece);
    else if (diff) hipLaunchKernelGGL((argmax_stream_kernel<1, true>), grid, block, 0, stream, p, w, piece);
    else hipLaunchKernelGGL((argmax_stream_kernel<1, false>), grid, block, 0, stream, p, w, piece);
    mk(K_TOPK_COLLECT);
    const dim3 fgrid((unsigned)((p.n + kArgThreads - 1) / kArgThreads));
    if (upd) hipLaunchKernelGGL((argmax_finish_kernel<true, true>), fgrid, block, 0, stream, p, w);
    else if (diff) hipLaunchKernelGGL((argmax_finish_kernel<true, false>), fgrid, block, 0, stream, p, w);
    else hipLaunchKernelGGL((argmax_finish_kernel<false, false>), fgrid, block, 0, stream, p, w);
    mk(K_TOPK_SELECT);
    return hipGetLastError();
}

}  // namespace

size_t topk_split_workspace_bytes(int32_t n, int64_t d, int64_t) { return layout(n, d, nullptr, nullptr); }

hipError_t launch_topk_split_reset(void *workspace, int32_t n, int64_t d, hipStream_t stream) {
    Ws w;
    layout(n, d, (char *)workspace, &w);
    // the histograms and the row records are the leading, contiguous part of the layout
    const size_t words = ((char *)w.slot_cnt - (char *)workspace) / sizeof(uint32_t);
    size_t blocks = (words + kCandThreads - 1) / kCandThreads;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(kCandThreads), 0, stream, (uint32_t *)workspace,
                       words);
    return hipGetLastError();
}

namespace {
// After the first collect pass: the second pass (after a warm start), count and emit.
hipError_t launch_after_collect(const TopkArgs &p, const Ws &w, hipStream_t stream, const Marker &mk) {
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    if (p.warm > 0) {
        launch_collect_any(p, w, kSecondPass, stream);
        mk(K_TOPK_REFINE);
    }
    const int spw = (int64_t)p.n * ((w.nslot + kCandWaves - 1) / kCandWaves) > 256 ? 2 : 1;
    const unsigned slot_blocks = (unsigned)((w.nslot + kCandWaves * spw - 1) / (kCandWaves * spw));
    const dim3 cgrid(slot_blocks + 1, (unsigned)p.n), block(kCandThreads);     // + 1: a row's rescue workgroup
#define EF21_CAND(KERNEL, GRID, DIFF, UPD)                                                               \
    do {                                                                                                 \
        if (spw == 2) hipLaunchKernelGGL((KERNEL<DIFF, UPD, 2>), GRID, block, 0, stream, p, w);          \
        else hipLaunchKernelGGL((KERNEL<DIFF, UPD, 1>), GRID, block, 0, stream, p, w);                   \
    } while (0)
    if (upd) EF21_CAND(cand_count_kernel, cgrid, true, true);
    else if (diff) EF21_CAND(cand_count_kernel, cgrid, true, false);
    else EF21_CAND(cand_count_kernel, cgrid, false, false);
    mk(K_TOPK_COUNT);
    if (upd) EF21_CAND(cand_emit_kernel, cgrid, true, true);
    else if (diff) EF21_CAND(cand_emit_kernel, cgrid, true, false);
    else EF21_CAND(cand_emit_kernel, cgrid, false, false);
#undef EF21_CAND
    mk(K_TOPK_EMIT);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_topk_split(const TopkArgs &p, void *workspace, hipStream_t stream, const Marker &mk) {
    Ws w;
    layout(p.n, p.d, (char *)workspace, &w);
    const bool diff = p.b != nullptr, upd = p.g_i != nullptr;
    if (upd && !diff) return hipErrorInvalidValue;
    if (p.warm < 0 || p.warm > kWarmSlots) return hipErrorInvalidValue;
    if (p.agg_start && (p.agg_shift < 0 || p.agg_shift > 11 || p.agg_nblk != ((p.d - 1) >> p.agg_shift) + 1 || p.k == 1))
        return hipErrorInvalidValue;
    if (p.k == 1) return launch_argmax(p, w, stream, mk);
    launch_collect_any(p, w, p.warm > 0 ? kWarmPass : kColdPass, stream);
    mk(K_TOPK_COLLECT);
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return st;
    return launch_after_collect(p, w, stream, mk);
}

int64_t topk_split_slots(int32_t n, int64_t d) {
    Ws w;
    plan(n, d, &w);
    return w.nslot;
}

hipError_t launch_topk_split_pair(const TopkArgs &plain, const TopkArgs &markov, void *ws_plain, void *ws_markov,
                                  void *norm_parts, hipStream_t stream, const Marker &mk) {
    if (plain.b || !markov.b || plain.a != markov.a || plain.n != markov.n || plain.d != markov.d ||
        plain.k != markov.k || plain.g_i || markov.g_i || plain.agg_start || markov.agg_start || plain.k < 2 ||
        plain.warm < 0 || plain.warm > kWarmSlots || markov.warm < 0 || markov.warm > kWarmSlots ||
        (plain.warm > 0) != (markov.warm > 0) || !norm_parts)
        return hipErrorInvalidValue;
    Ws wp, wm;
    layout(plain.n, plain.d, (char *)ws_plain, &wp);
    layout(markov.n, markov.d, (char *)ws_markov, &wm);
    const bool vec4 = (markov.d % 4 == 0) && ((uintptr_t)markov.a % 16 == 0) && ((uintptr_t)markov.b % 16 == 0);
    const bool warm = markov.warm > 0;
    const dim3 grid((unsigned)wm.G, (unsigned)markov.n), block(kBlk);
    double2 *norms = (double2 *)norm_parts;
    const bool two_per_cu = wm.G * markov.n > 256;      // steps per group: see launch_collect
#define EF21_PAIR(VEC, WARM, U) \
    hipLaunchKernelGGL((split_collect_pair_kernel<VEC, WARM, U>), grid, block, 0, stream, markov, wm, plain.warm, wp, norms)
    if (vec4 && warm && two_per_cu) EF21_PAIR(4, true, 1);
    else if (vec4 && warm) EF21_PAIR(4, true, 2);
    else if (vec4 && two_per_cu) EF21_PAIR(4, false, 1);
    else if (vec4) EF21_PAIR(4, false, 2);
    else if (warm) EF21_PAIR(1, true, 2);
    else EF21_PAIR(1, false, 2);
#undef EF21_PAIR
    mk(K_TOPK_COLLECT);
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return st;
    st = launch_after_collect(plain, wp, stream, mk);
    if (st != hipSuccess) return st;
    return launch_after_collect(markov, wm, stream, mk);
}

}  // namespace ef21
