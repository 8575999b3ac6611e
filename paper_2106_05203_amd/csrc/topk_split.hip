// Batched Top-k (Section 2.1 of the EF21 paper) for long rows: many workgroups per row, the row
// itself read ONCE.
//
// Same selection rule as the one-workgroup kernel (31-bit magnitude key, ties to the lower index,
// ascending output).  Pipeline:
//
//   collect   Every workgroup first looks at the same fixed sample of its row (32 evenly spaced
//             pieces of 256 entries), finds in LDS a key `key_lo` that, with overwhelming
//             probability, at least k entries of the row reach, and then streams its part of the
//             row.  Each wavefront owns a contiguous piece of the row and appends the entries
//             with key >= key_lo ("candidates", a few per cent of the row) in position order to
//             its own slot of the workspace.  No atomics, no fences, no inter-workgroup traffic.
//   then, on the candidates only, either
//   select    (small k) one workgroup per row: candidate keys into LDS, radix select there, ordered
//             emission of the k kept entries (+ line 6 of Algorithm 2); or
//   hist x2, count, emit   (large k) the same steps spread over several workgroups per row,
//             chained by kernel boundaries: a kernel merges its LDS histograms into the row's
//             global one with a few atomics per bin, the NEXT kernel's workgroups each scan the
//             merged histogram in their prologue.  The candidates' keys lie at or above key_lo and
//             the threshold key T a little above it, so the two digits are taken from key - key_lo:
//             12 bits from bit 11 upwards (a window of one octave; keys beyond it share the last
//             bin), then the low 11 bits.
//
// The estimate can be wrong (fewer than k candidates, or T beyond the window); the row is then selected by the exact
// one-workgroup algorithm on the original data (inside `select`, or by an extra workgroup of the
// `count` kernel), so the result never depends on the sample.  Slots have the capacity of their piece, so any input fits.
#include <cmath>

#include "topk_row_impl.h"

namespace ef21 {
namespace {

constexpr int kBlk = kRowThreads;            // collect / select / rescue workgroups
constexpr int kBlkWaves = kBlk / kWave;
constexpr int kSample = 8192;                // sampled entries per row
constexpr int kSamplePer = kSample / kBlk;
constexpr int kPieceLen = 256, kPieces = kSample / kPieceLen;
constexpr int kMaxSlots = 4096;              // slots (wavefront pieces) per row
constexpr int kSelCap = 28672;               // candidate keys the select kernel holds in LDS
// Rows expected to keep more candidates than this take the many-workgroup stages: their four launches cost about
// 28 us whatever k is, the one-workgroup select grows with the candidates and passes that at about 12 000.
constexpr int kSelectMax = 12288;
constexpr int kCandThreads = 1024;           // count / emit workgroups (large k): one wavefront per slot
constexpr int kCandWaves = kCandThreads / kWave;
constexpr int kHistThreads = 512;            // candidate histogram workgroups (large k)
constexpr int kCandBlocks = 16;              // ... of which each row gets this many
constexpr int kBins1 = 1 << kBits1, kBins2 = 1 << kBits2, kBins3 = 1 << kBits3;
constexpr int kBitsA = 12, kBitsB = 11;        // large k: digits of key - key_lo
constexpr int kBinsA = 1 << kBitsA, kBinsB = 1 << kBitsB;

struct RowInfo {
    uint32_t failed, M;       // the estimate failed (see above); number of candidates
    uint32_t bin_a, need_a;   // first digit of T - key_lo; entries still needed from that bin
    uint32_t T, q;            // threshold key; number of entries equal to T to keep
    uint32_t key_lo, pad;     // lower bound of the candidate keys (from collect)
};

struct Ws {
    uint32_t *hist_a, *hist_b;            // [n][kBinsA], [n][kBinsB], kept zero between calls
    RowInfo *info;                        // [n]
    uint32_t *slot_cnt, *slot_gt, *slot_eq;   // [n][nslot]
    int32_t *cand_idx;                    // [n][nslot][L]
    float *cand_val;
    float *cand_new;                      // [n][nslot][L]  b + v of the candidate (new g_i entry if kept)
    int64_t L;                            // entries per wavefront piece = slot capacity
    int64_t nslot;                        // pieces per row
    int64_t G;                            // collect workgroups per row
};

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

void plan(int32_t n, int64_t d, Ws *w) {
    // one 1024-thread workgroup per CU, two (in two rounds: the kernel's registers let one be resident) for inputs
    // of 2^26 entries and more: measured on 20 x 10^6 (37.7 against 38.2 us per call) and 8 x 11.2 * 10^6 (168 against
    // 162 us per collect pass)
    int64_t max_g = ((int64_t)n * d >= ((int64_t)1 << 26) ? 512 : 256) / n;
    if (max_g < 1) max_g = 1;
    if (max_g > kMaxSlots / kBlkWaves) max_g = kMaxSlots / kBlkWaves;
    int64_t g = (d + kBlkWaves * 2048 - 1) / (kBlkWaves * 2048);   // at least 2048 entries per piece
    if (g > max_g) g = max_g;
    if (g < 1) g = 1;
    const int64_t pieces = g * kBlkWaves;
    int64_t L = (d + pieces - 1) / pieces;
    L = (L + 1023) / 1024 * 1024;            // whole load groups (4 steps of 64 lanes x 4 entries)
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
    char *h2 = take(sizeof(uint32_t) * (size_t)n * kBinsA);
    char *h3 = take(sizeof(uint32_t) * (size_t)n * kBinsB);
    char *inf = take(sizeof(RowInfo) * (size_t)n);
    const size_t slots = sizeof(uint32_t) * (size_t)n * tmp.nslot;
    char *s0 = take(slots), *s1 = take(slots), *s2 = take(slots);
    char *ci = take(sizeof(int32_t) * (size_t)n * tmp.nslot * tmp.L);
    char *cv = take(sizeof(float) * (size_t)n * tmp.nslot * tmp.L);
    char *cn = take(sizeof(float) * (size_t)n * tmp.nslot * tmp.L);
    if (w) {
        *w = tmp;
        w->hist_a = (uint32_t *)h2; w->hist_b = (uint32_t *)h3;
        w->info = (RowInfo *)inf;
        w->slot_cnt = (uint32_t *)s0; w->slot_gt = (uint32_t *)s1; w->slot_eq = (uint32_t *)s2;
        w->cand_idx = (int32_t *)ci; w->cand_val = (float *)cv; w->cand_new = (float *)cn;
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

// Per-wavefront staging ring in LDS: candidates are appended here and leave for the slot in global
// memory 64 at a time, as one full-width store per array, instead of as many scattered 4-byte stores.
// With UPDATE a candidate also carries b + v, the value g_i takes at its position if it is kept.
constexpr uint32_t kRing = 128;              // entries of a staging ring (power of two, >= 128)
struct StageRing {
    int32_t idx[kRing];
    float val[kRing];
    float nxt[kRing];
};

struct SlotPtrs {
    int32_t *idx;
    float *val;
    float *nxt;
};

// Writes the entries [flushed, flushed + count) of the ring (count <= 64) to the slot.
template <bool UPDATE>
__device__ __forceinline__ void ring_to_slot(const StageRing &ring, uint32_t flushed, uint32_t count, int lane,
                                             const SlotPtrs &slot) {
    if ((uint32_t)lane < count) {
        slot.idx[flushed + lane] = ring.idx[(flushed + lane) & (kRing - 1)];
        slot.val[flushed + lane] = ring.val[(flushed + lane) & (kRing - 1)];
        if (UPDATE) slot.nxt[flushed + lane] = ring.nxt[(flushed + lane) & (kRing - 1)];
    }
}

// Appends the candidates among one step's entries (VEC per lane, lane-major order) to the slot.
// FULL: every entry of the step lies inside the piece, no bounds checks.  bv: the subtracted values.
// cnt = candidates so far, flushed = how many of them are already in global memory (cnt - flushed < 64
// between calls; both are uniform over the wavefront).
template <int VEC, bool FULL, bool UPDATE>
__device__ __forceinline__ void append_candidates(const float (&v)[VEC], const float (&bv)[VEC], int64_t e0,
                                                  int64_t hi, uint32_t key_lo, StageRing &ring, int lane,
                                                  const SlotPtrs &slot, uint32_t &cnt, uint32_t &flushed) {
    bool c[VEC];
    uint32_t below = 0, all = 0;
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        c[t] = (FULL || e0 + t < hi) && mag_key(v[t]) >= key_lo;
        const uint64_t m = __ballot(c[t]);
        below += lanes_below(m);
        all += popc64(m);
    }
    if (all == 0) return;
    uint32_t pos = cnt + below;
    if (all > 64) {        // a dense step would not fit the ring: drain it, then store directly
        ring_to_slot<UPDATE>(ring, flushed, cnt - flushed, lane, slot);
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            if (c[t]) {
                slot.idx[pos] = (int32_t)(e0 + t);
                slot.val[pos] = v[t];
                if (UPDATE) slot.nxt[pos] = bv[t] + v[t];
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
            ring.idx[pos & (kRing - 1)] = (int32_t)(e0 + t);
            ring.val[pos & (kRing - 1)] = v[t];
            if (UPDATE) ring.nxt[pos & (kRing - 1)] = bv[t] + v[t];
            ++pos;
        }
    }
    cnt += all;
    if (cnt - flushed > kRing - 64) {        // keep room for the next step's candidates (at most 64)
        __builtin_amdgcn_wave_barrier();
        ring_to_slot<UPDATE>(ring, flushed, 64, lane, slot);
        flushed += 64;
    }
}

// Writes what is left in the ring at the end of a piece.
template <bool UPDATE>
__device__ __forceinline__ void drain_ring(const StageRing &ring, uint32_t flushed, uint32_t cnt, int lane,
                                           const SlotPtrs &slot) {
    __builtin_amdgcn_wave_barrier();
    for (; flushed < cnt; flushed += 64)
        ring_to_slot<UPDATE>(ring, flushed, cnt - flushed < 64 ? cnt - flushed : 64, lane, slot);
}

// A wavefront walks its piece in steps of 64*VEC entries (VEC = 4 needs 16-byte aligned rows), four
// steps per group.  Whole groups are loaded without any bounds check so that all loads of a group
// are in flight together; only the last piece of a row has a checked tail.
template <int VEC, bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kBlk) void split_collect_kernel(TopkArgs p, Ws w) {
    static_assert(DIFF || !UPDATE, "the update needs the subtracted g_i");
    __shared__ RowShared s;
    __shared__ StageRing rings[kBlkWaves];
    const int64_t row = blockIdx.y, d = p.d;
    const float *a = p.a + row * d;
    const float *b = DIFF ? p.b + row * d : nullptr;
    const uint32_t key_lo = estimate_key_lo<DIFF>(s, a, b, d, p.k);
    if (blockIdx.x == 0 && threadIdx.x == 0) w.info[row].key_lo = key_lo;

    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int64_t slot_no = (int64_t)blockIdx.x * kBlkWaves + wave;
    if (slot_no < w.nslot) {
        StageRing &ring = rings[wave];
        const int64_t lo = slot_no * w.L;
        const int64_t hi = lo + w.L < d ? lo + w.L : d;
        const int64_t slot_at = (row * w.nslot + slot_no) * w.L;
        const SlotPtrs slot{w.cand_idx + slot_at, w.cand_val + slot_at, w.cand_new + slot_at};
        uint32_t cnt = 0, flushed = 0;
        constexpr int kStep = kWave * VEC, kUnroll = 4, kGroup = kStep * kUnroll;
        int64_t base = lo;
        for (; base + kGroup <= hi; base += kGroup) {
            float v[kUnroll][VEC], bv[kUnroll][VEC];
            if constexpr (VEC == 4) {
                float4 va[kUnroll], vb[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    va[u] = stream_load4(a + base + u * kStep + lane * 4);
                    if constexpr (DIFF) vb[u] = stream_load4(b + base + u * kStep + lane * 4);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    v[u][0] = va[u].x; v[u][1] = va[u].y; v[u][2] = va[u].z; v[u][3] = va[u].w;
                    if constexpr (DIFF) {
                        bv[u][0] = vb[u].x; bv[u][1] = vb[u].y; bv[u][2] = vb[u].z; bv[u][3] = vb[u].w;
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    v[u][0] = stream_load(a + base + u * kStep + lane);
                    if constexpr (DIFF) bv[u][0] = stream_load(b + base + u * kStep + lane);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
                for (int t = 0; t < VEC; ++t) {
                    if constexpr (DIFF) v[u][t] -= bv[u][t];
                    else bv[u][t] = 0.f;
                }
                append_candidates<VEC, true, UPDATE>(v[u], bv[u], base + u * kStep + lane * VEC, hi, key_lo, ring,
                                                     lane, slot, cnt, flushed);
            }
        }
        for (; base < hi; base += kStep) {           // checked tail, entry by entry
            const int64_t e0 = base + lane * VEC;
            float v[VEC], bv[VEC];
#pragma unroll
            for (int t = 0; t < VEC; ++t) {
                v[t] = e0 + t < hi ? a[e0 + t] : 0.f;
                bv[t] = DIFF && e0 + t < hi ? b[e0 + t] : 0.f;
                v[t] -= bv[t];
            }
            append_candidates<VEC, false, UPDATE>(v, bv, e0, hi, key_lo, ring, lane, slot, cnt, flushed);
        }
        drain_ring<UPDATE>(ring, flushed, cnt, lane, slot);
        if (lane == 0) w.slot_cnt[row * w.nslot + slot_no] = cnt;
    }
}

// ---------------------------------------------------------------- select (small k): one workgroup per row
// Each wavefront owns a contiguous range of the row's slots, hence a contiguous range of the flat list
// of candidates.  With W = the row's largest slot count rounded up to a power of two, a slot is cut into
// units of min(W, 64) entries: one load instruction serves 64 / W slots if W < 64 (lane = slot * W +
// entry) or one of the W / 64 steps of a slot otherwise; either way the lanes, the units of a batch and
// the batches follow the candidate order, and kSlotBatch units are in flight together.  Rows with a slot
// above kMaxUnitSlot candidates are walked slot by slot instead.
constexpr int kSlotBatch = 8;
constexpr uint32_t kMaxUnitSlot = 256;

template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kBlk) void split_select_kernel(TopkArgs p, Ws w) {
    __shared__ RowShared s;
    __shared__ uint32_t off[kMaxSlots + 1];      // exclusive prefix of the slot counts
    extern __shared__ uint32_t keys[];           // [kSelCap]
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    const int nslot = (int)w.nslot;
    const uint32_t *slot_cnt = w.slot_cnt + row * w.nslot;

    // exclusive scan of the slot counts (four consecutive slots per thread) and their maximum
    constexpr int kPer = kMaxSlots / kBlk;
    uint32_t c[kPer], mine = 0, largest = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int sl = tid * kPer + j;
        c[j] = sl < nslot ? slot_cnt[sl] : 0u;
        mine += c[j];
        largest = c[j] > largest ? c[j] : largest;
    }
    const uint32_t incl = wave_inclusive_scan(mine);
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const uint32_t other = __shfl_xor(largest, o, kWave);
        largest = other > largest ? other : largest;
    }
    if (lane == kWave - 1) s.wave_a[wave] = incl;
    if (lane == 0) s.wave_b[wave] = largest;
    __syncthreads();
    uint32_t run = incl - mine;
    for (int v = 0; v < wave; ++v) run += s.wave_a[v];
    largest = 0;
    for (int v = 0; v < kBlkWaves; ++v) largest = s.wave_b[v] > largest ? s.wave_b[v] : largest;
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

    const float *cand_val = w.cand_val + row * w.nslot * w.L;
    const int32_t *cand_idx = w.cand_idx + row * w.nslot * w.L;
    const float *cand_new = w.cand_new + row * w.nslot * w.L;
    // this wavefront's slots [s0, s1) and candidates [lo, hi)
    const int per_wave = (nslot + kBlkWaves - 1) / kBlkWaves;
    const int s0 = wave * per_wave < nslot ? wave * per_wave : nslot;
    const int s1 = s0 + per_wave < nslot ? s0 + per_wave : nslot;
    const uint32_t lo = off[s0], hi = off[s1];
    // the units (see above): either several slots per unit or several units per slot
    uint32_t W = 1;
    while (W < kMaxUnitSlot && W < largest) W <<= 1;
    const int slots_per_unit = W < (uint32_t)kWave ? kWave / (int)W : 1;    // slots served by one unit
    const int units_per_slot = W > (uint32_t)kWave ? (int)W / kWave : 1;    // units a slot is cut into
    const int lanes_per_slot = W < (uint32_t)kWave ? (int)W : kWave;
    const int my_slot = lane / lanes_per_slot;        // slot of this lane inside a unit
    const uint32_t my_e = (uint32_t)(lane % lanes_per_slot);
    const bool crowded = largest > kMaxUnitSlot;
    const int n_units = (s1 - s0 + slots_per_unit - 1) / slots_per_unit * units_per_slot;
    // unit t of this wavefront -> (slot, entry of this lane); slot >= s1 marks a lane without a slot
    auto unit_slot = [&](int t) { return s0 + (t / units_per_slot) * slots_per_unit + my_slot; };
    auto unit_entry = [&](int t) { return (uint32_t)(t % units_per_slot) * (uint32_t)kWave + my_e; };

    // candidate keys into LDS
    if (!crowded) {
        for (int t0 = 0; t0 < n_units; t0 += kSlotBatch) {
            float v[kSlotBatch];
            uint32_t at_key[kSlotBatch];
            bool in[kSlotBatch];
#pragma unroll
            for (int u = 0; u < kSlotBatch; ++u) {
                const int sl = unit_slot(t0 + u);
                const uint32_t j = unit_entry(t0 + u);
                const int slc = sl < s1 ? sl : s1 - 1;
                const uint32_t first = off[slc], cnt = off[slc + 1] - first;
                in[u] = t0 + u < n_units && sl < s1 && j < cnt;
                at_key[u] = first + j;
                v[u] = cand_val[(int64_t)slc * w.L + (in[u] ? j : 0u)];     // clamped: no load behind a branch
            }
#pragma unroll
            for (int u = 0; u < kSlotBatch; ++u)
                if (in[u]) keys[at_key[u]] = mag_key(v[u]);
        }
    } else {
        for (int sl = s0; sl < s1; ++sl) {
            const uint32_t first = off[sl], cnt = off[sl + 1] - first;
            for (uint32_t j0 = 0; j0 < cnt; j0 += kWave * kSlotBatch) {
                float v[kSlotBatch];
#pragma unroll
                for (int u = 0; u < kSlotBatch; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    v[u] = cand_val[(int64_t)sl * w.L + (j < cnt ? j : 0u)];
                }
#pragma unroll
                for (int u = 0; u < kSlotBatch; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    if (j < cnt) keys[first + j] = mag_key(v[u]);
                }
            }
        }
    }
    __syncthreads();

    // Radix select over the keys in LDS.  All candidates have key >= key_lo and the threshold lies a little above
    // it, so the first digit is taken from key - key_lo (12 bits from bit 11, larger differences in the last bin):
    // the candidates spread over hundreds of bins, where the leading bits of the keys themselves would put them
    // all into a handful (LDS atomics on the same address are served one after the other).  Then either the
    // bin's entries ranked against one another (at most kRankMax of them; their place in the candidate list is
    // their order among equal keys) or the low 11 bits by a second histogram.  A threshold in the last bin
    // (k tiny against the candidates) is found on the keys' own digits instead.
    uint32_t prefix = 0, need = (uint32_t)p.k;
    bool found = false;
    {
        const uint32_t key_lo = w.info[row].key_lo;
        auto digit_a = [&](uint32_t key) {
            const uint32_t rel = (key - key_lo) >> kBitsB;
            return rel < (uint32_t)kBinsA - 1u ? rel : (uint32_t)kBinsA - 1u;
        };
        static_assert(kBinsA == kBins1, "the first relative digit uses the 12-bit histogram");
        for (int i = tid; i < kBinsA; i += kBlk) s.hist[i] = 0u;
        __syncthreads();
        for (uint32_t j = tid; j < M; j += kBlk) atomicAdd(&s.hist[digit_a(keys[j])], 1u);
        __syncthreads();
        select_bin(s, kBinsA, need);
        const uint32_t bin_a = s.bin, need_a = s.need, in_bin = s.hist[bin_a];
        if (tid == 0) s.ncand = 0u;
        if (tid < kRankMax) s.cand_rank[tid] = 0u;
        __syncthreads();
        if (bin_a != (uint32_t)kBinsA - 1u) {
            found = true;
            if (in_bin <= (uint32_t)kRankMax) {
                for (uint32_t j = tid; j < M; j += kBlk) {
                    const uint32_t key = keys[j];
                    if (digit_a(key) == bin_a) {
                        const uint32_t at = atomicAdd(&s.ncand, 1u);
                        s.cand_key[at] = key;
                        s.cand_idx[at] = j;
                    }
                }
                __syncthreads();
                rank_gathered(s, need_a);
                prefix = s.bin;
                need = s.need;
            } else {
                for (int i = tid; i < kBinsB; i += kBlk) s.hist[i] = 0u;
                __syncthreads();
                for (uint32_t j = tid; j < M; j += kBlk) {
                    const uint32_t key = keys[j];
                    if (digit_a(key) == bin_a) atomicAdd(&s.hist[(key - key_lo) & ((uint32_t)kBinsB - 1u)], 1u);
                }
                __syncthreads();
                select_bin(s, kBinsB, need_a);
                prefix = key_lo + ((bin_a << kBitsB) | s.bin);
                need = s.need;
            }
            __syncthreads();
        }
    }
    if (!found) {
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
            const uint32_t in_bin = s.hist[s.bin];
            if (tid == 0) s.ncand = 0u;
            if (tid < kRankMax) s.cand_rank[tid] = 0u;
            __syncthreads();
            if (pass == 0 && in_bin <= (uint32_t)kRankMax) {
                for (uint32_t j = tid; j < M; j += kBlk) {
                    const uint32_t key = keys[j];
                    if ((key >> (kBits2 + kBits3)) == prefix) {
                        const uint32_t at = atomicAdd(&s.ncand, 1u);
                        s.cand_key[at] = key;
                        s.cand_idx[at] = j;
                    }
                }
                __syncthreads();
                rank_gathered(s, need);
                prefix = s.bin;
                need = s.need;
                break;
            }
        }
    }
    const uint32_t T = prefix, q = need;

    // ordered emission: counts of this wavefront's range, prefix over the wavefronts ...
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
    float *g_row = UPDATE ? p.g_i + row * p.d : nullptr;
    // one step of the emission over 64 lanes in candidate order; `in` marks lanes that hold a candidate
    auto emit_step = [&](bool in, uint32_t key, int32_t e, float v, float nx) {
        const bool gt = in && key > T, eq = in && key == T;
        const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
        const uint32_t eq_below = eq_run + lanes_below(m_eq);
        const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
        if (gt || (eq && eq_below < q)) {
            const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
            out_idx[pos] = e;
            out_val[pos] = v;
            if (UPDATE) g_row[e] = nx;          // Algorithm 2, line 6
        }
        const uint32_t eq_next = eq_run + popc64(m_eq);
        out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_run < q ? eq_run : q));
        eq_run = eq_next;
    };
    // ... then the slots in order: (position, value[, new g_i entry]) of a whole batch are loaded, then the
    // kept ones written
    if (!crowded) {
        for (int t0 = 0; t0 < n_units; t0 += kSlotBatch) {
            int32_t e[kSlotBatch];
            float v[kSlotBatch], nx[kSlotBatch];
            uint32_t key[kSlotBatch];
            bool in[kSlotBatch];
#pragma unroll
            for (int u = 0; u < kSlotBatch; ++u) {
                const int sl = unit_slot(t0 + u);
                const uint32_t j = unit_entry(t0 + u);
                const int slc = sl < s1 ? sl : s1 - 1;
                const uint32_t first = off[slc], cnt = off[slc + 1] - first;
                in[u] = t0 + u < n_units && sl < s1 && j < cnt;
                const int64_t at = (int64_t)slc * w.L + (in[u] ? j : 0u);
                e[u] = cand_idx[at];
                v[u] = cand_val[at];
                nx[u] = UPDATE ? cand_new[at] : 0.f;
                key[u] = in[u] ? keys[first + j] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kSlotBatch; ++u) emit_step(in[u], key[u], e[u], v[u], nx[u]);
        }
    } else {
        for (int sl = s0; sl < s1; ++sl) {
            const uint32_t first = off[sl], cnt = off[sl + 1] - first;
            for (uint32_t j0 = 0; j0 < cnt; j0 += kWave * kSlotBatch) {
                int32_t e[kSlotBatch];
                float v[kSlotBatch], nx[kSlotBatch];
#pragma unroll
                for (int u = 0; u < kSlotBatch; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    const int64_t at = (int64_t)sl * w.L + (j < cnt ? j : 0u);
                    e[u] = cand_idx[at];
                    v[u] = cand_val[at];
                    nx[u] = UPDATE ? cand_new[at] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < kSlotBatch; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    emit_step(j < cnt, j < cnt ? keys[first + j] : 0u, e[u], v[u], nx[u]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------- candidate stages (large k)
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

// Digit selection over the row's merged histogram (written by the previous kernel): largest bin b
// with count(bins > b) < need <= count(bins >= b).  lds_out[0] = b, lds_out[1] = need - count(bins > b).
template <int NBINS, int THREADS>
__device__ void select_digit(const uint32_t *hist, uint32_t need, uint32_t *lds_wave, uint32_t *lds_out) {
    constexpr int PER = NBINS >= THREADS ? NBINS / THREADS : 1;      // bins per thread, walked from the top
    static_assert(NBINS % PER == 0 && NBINS / PER <= THREADS, "histogram must divide over the workgroup");
    const bool active = (int)threadIdx.x < NBINS / PER;
    uint32_t h[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[j] = active ? hist[NBINS - 1 - ((int)threadIdx.x * PER + j)] : 0u;
        mine += h[j];
    }
    uint32_t total;
    const uint32_t above = cand_block_scan<THREADS>(mine, lds_wave, &total);
    if (active && above < need && need <= above + mine) {
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

__device__ void zero_global_hist(uint32_t *hist, int bins) {
    for (int i = threadIdx.x; i < bins; i += blockDim.x) hist[i] = 0u;
}

// Digit STAGE (1 or 2) of the radix select over the candidates' key - key_lo, kCandBlocks workgroups per
// row (few, so that the merge below costs a few atomics per bin).  Prologue: stage 1 adds up the slot
// counts (fewer than k candidates: the estimate failed); stage 2 selects the first digit from the merged
// histogram (the last bin, which also holds every key beyond the window, cannot be resolved: failed).
// Body: LDS histogram of this stage's digit over the workgroup's slots, four slots in flight per
// wavefront, then merged into the row's global histogram.
// A failed row is left alone by the later kernels, except for one extra workgroup of the count kernel
// that selects it by the exact one-workgroup algorithm on the original data.
template <int STAGE>
__global__ __launch_bounds__(kHistThreads) void cand_hist_kernel(TopkArgs p, Ws w) {
    static_assert(STAGE == 1 || STAGE == 2, "two digits");
    constexpr int NB = STAGE == 1 ? kBinsA : kBinsB;
    __shared__ uint32_t hist[NB];
    __shared__ uint32_t lds_wave[kHistThreads / kWave], lds_out[2];
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    const uint32_t *slot_cnt = w.slot_cnt + row * w.nslot;
    const uint32_t key_lo = info->key_lo;
    uint32_t bin_a = 0;
    if constexpr (STAGE == 1) {
        uint32_t mine = 0, M;
        for (int64_t sl = threadIdx.x; sl < w.nslot; sl += kHistThreads) mine += slot_cnt[sl];
        (void)cand_block_scan<kHistThreads>(mine, lds_wave, &M);
        const bool failed = M < (uint32_t)p.k;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            info->failed = failed ? 1u : 0u;
            info->M = M;
        }
        if (failed) return;
    } else {
        if (info->failed) return;
        select_digit<kBinsA, kHistThreads>(w.hist_a + row * kBinsA, (uint32_t)p.k, lds_wave, lds_out);
        bin_a = lds_out[0];
        const bool failed = bin_a == (uint32_t)kBinsA - 1u;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            info->bin_a = bin_a;
            info->need_a = lds_out[1];
            if (failed) info->failed = 1u;
        }
        if (failed) return;
    }
    for (int i = threadIdx.x; i < NB; i += kHistThreads) hist[i] = 0u;
    __syncthreads();
    // kInFlight slots of the wavefront at a time, kSteps steps of 64 candidates of each: all loads of such a
    // round are issued before the first is used (a slot usually holds fewer than kSteps * 64 candidates)
    constexpr int kInFlight = 8, kSteps = 4;
    const int64_t stride = (int64_t)kCandBlocks * (kHistThreads / kWave);
    for (int64_t sl0 = (int64_t)blockIdx.x * (kHistThreads / kWave) + wave; sl0 < w.nslot; sl0 += stride * kInFlight) {
        uint32_t cnt[kInFlight], most = 0;
        const float *val[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int64_t sl = sl0 + u * stride;
            cnt[u] = sl < w.nslot ? slot_cnt[sl] : 0u;
            val[u] = w.cand_val + (row * w.nslot + (sl < w.nslot ? sl : 0)) * w.L;
            most = cnt[u] > most ? cnt[u] : most;
        }
        for (uint32_t j0 = 0; j0 < most; j0 += kWave * kSteps) {
            float v[kSteps][kInFlight];
#pragma unroll
            for (int q = 0; q < kSteps; ++q)
#pragma unroll
                for (int u = 0; u < kInFlight; ++u) {
                    const uint32_t j = j0 + q * kWave + lane;
                    v[q][u] = val[u][j < cnt[u] ? j : 0u];            // clamped: no load behind a branch
                }
#pragma unroll
            for (int q = 0; q < kSteps; ++q)
#pragma unroll
                for (int u = 0; u < kInFlight; ++u) {
                    const uint32_t j = j0 + q * kWave + lane;
                    if (j >= cnt[u]) continue;
                    const uint32_t rel = mag_key(v[q][u]) - key_lo;       // candidates have key >= key_lo
                    const uint32_t a = rel >> kBitsB < (uint32_t)kBinsA - 1u ? rel >> kBitsB : (uint32_t)kBinsA - 1u;
                    if (STAGE == 1) atomicAdd(&hist[a], 1u);
                    else if (a == bin_a) atomicAdd(&hist[rel & (kBinsB - 1)], 1u);
                }
        }
    }
    __syncthreads();
    uint32_t *merged = STAGE == 1 ? w.hist_a + row * kBinsA : w.hist_b + row * kBinsB;
    for (int b = threadIdx.x; b < NB; b += kHistThreads) {
        const uint32_t c = hist[b];
        if (c) atomicAdd(merged + b, c);
    }
}

// One wavefront per slot.  Prologue: threshold key T and tie quota q from the third digit's
// histogram.  Body: the slot's number of candidates above T and equal to T.
template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kCandThreads) void cand_count_kernel(TopkArgs p, Ws w) {
    static_assert(kCandThreads == kRowThreads, "the rescue workgroup runs the one-workgroup algorithm");
    __shared__ RowShared rs;
    __shared__ uint32_t lds_wave[kCandWaves], lds_out[2];
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    RowInfo *info = w.info + row;
    if (blockIdx.x == gridDim.x - 1) {               // the rescue workgroup (DIFF, UPDATE matter here only)
        if (info->failed) {
            zero_global_hist(w.hist_a + row * kBinsA, kBinsA);     // left behind if stage 2 declared the failure
            row_topk<DIFF, UPDATE>(rs, p, row);
        }
        return;
    }
    if (info->failed) return;
    select_digit<kBinsB, kCandThreads>(w.hist_b + row * kBinsB, info->need_a, lds_wave, lds_out);
    const uint32_t T = info->key_lo + ((info->bin_a << kBitsB) | lds_out[0]);
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            info->T = T;
            info->q = lds_out[1];
        }
        zero_global_hist(w.hist_a + row * kBinsA, kBinsA);     // consumed by stage 2
    }
    const int64_t sl = (int64_t)blockIdx.x * kCandWaves + wave;
    if (sl >= w.nslot) return;
    const uint32_t cnt = w.slot_cnt[row * w.nslot + sl];
    const float *slot_val = w.cand_val + (row * w.nslot + sl) * w.L;
    uint32_t n_gt = 0, n_eq = 0;
    constexpr int kSteps = 4;
    for (uint32_t j0 = 0; j0 < cnt; j0 += kWave * kSteps) {
        float v[kSteps];
#pragma unroll
        for (int q = 0; q < kSteps; ++q) {
            const uint32_t j = j0 + q * kWave + lane;
            v[q] = slot_val[j < cnt ? j : 0u];
        }
#pragma unroll
        for (int q = 0; q < kSteps; ++q) {
            const uint32_t j = j0 + q * kWave + lane;
            const uint32_t key = mag_key(v[q]);
            n_gt += popc64(__ballot(j < cnt && key > T));
            n_eq += popc64(__ballot(j < cnt && key == T));
        }
    }
    if (lane == 0) {
        w.slot_gt[row * w.nslot + sl] = n_gt;
        w.slot_eq[row * w.nslot + sl] = n_eq;
    }
}

// Ordered emission, one wavefront per slot.  The workgroup first adds up the counts of all slots of its
// row before its own (at most kMaxSlots of them), which gives its output offset and the number of ties
// already used; a wavefront then adds the counts of the workgroup's earlier slots.
template <bool UPDATE>
__global__ __launch_bounds__(kCandThreads) void cand_emit_kernel(TopkArgs p, Ws w) {
    __shared__ uint32_t before_gt[kCandWaves], before_eq[kCandWaves], own_gt[kCandWaves], own_eq[kCandWaves];
    const int64_t row = blockIdx.y;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const RowInfo *info = w.info + row;
    if (info->failed) return;                                                     // the whole workgroup
    if (blockIdx.x == 0) zero_global_hist(w.hist_b + row * kBinsB, kBinsB);       // consumed by count
    const int64_t sl0 = (int64_t)blockIdx.x * kCandWaves, sl = sl0 + wave;
    const bool active = sl < w.nslot;
    const uint32_t T = info->T, q = info->q;
    const uint32_t *slot_gt = w.slot_gt + row * w.nslot, *slot_eq = w.slot_eq + row * w.nslot;
    uint32_t gt_part = 0, eq_part = 0;
    for (int64_t t = threadIdx.x; t < sl0; t += kCandThreads) {
        gt_part += slot_gt[t];
        eq_part += slot_eq[t];
    }
    const uint32_t mine_gt = active ? slot_gt[sl] : 0u, mine_eq = active ? slot_eq[sl] : 0u;
    const uint32_t cnt = active ? w.slot_cnt[row * w.nslot + sl] : 0u;
    gt_part = wave_sum_u32(gt_part);
    eq_part = wave_sum_u32(eq_part);
    if (lane == 0) {
        before_gt[wave] = gt_part;
        before_eq[wave] = eq_part;
        own_gt[wave] = mine_gt;
        own_eq[wave] = mine_eq;
    }
    __syncthreads();
    if (!active) return;
    uint32_t gt_run = 0, eq_run = 0;
    for (int v = 0; v < kCandWaves; ++v) {
        gt_run += before_gt[v] + (v < wave ? own_gt[v] : 0u);
        eq_run += before_eq[v] + (v < wave ? own_eq[v] : 0u);
    }
    uint32_t out_run = gt_run + (eq_run < q ? eq_run : q);
    const int32_t *slot_idx = w.cand_idx + (row * w.nslot + sl) * w.L;
    const float *slot_val = w.cand_val + (row * w.nslot + sl) * w.L;
    const float *slot_new = w.cand_new + (row * w.nslot + sl) * w.L;
    int32_t *out_idx = p.out_idx + row * p.k;
    float *out_val = p.out_val + row * p.k;
    constexpr int kSteps = 4;
    for (uint32_t j0 = 0; j0 < cnt; j0 += kWave * kSteps) {
        float v[kSteps], nx[kSteps];
        int32_t e[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const uint32_t j = j0 + s * kWave + lane;
            const uint32_t jc = j < cnt ? j : 0u;                // clamped: no load behind a branch
            v[s] = slot_val[jc];
            e[s] = slot_idx[jc];
            nx[s] = UPDATE ? slot_new[jc] : 0.f;
        }
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const uint32_t j = j0 + s * kWave + lane;
            const bool in = j < cnt;
            const uint32_t key = mag_key(v[s]);
            const bool gt = in && key > T, eq = in && key == T;
            const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
            const uint32_t eq_below = eq_run + lanes_below(m_eq);
            const uint32_t ties_before = (eq_below < q ? eq_below : q) - (eq_run < q ? eq_run : q);
            if (gt || (eq && eq_below < q)) {
                const uint32_t pos = out_run + lanes_below(m_gt) + ties_before;
                out_idx[pos] = e[s];
                out_val[pos] = v[s];
                if (UPDATE) (p.g_i + row * p.d)[e[s]] = nx[s];   // Algorithm 2, line 6
            }
            const uint32_t eq_next = eq_run + popc64(m_eq);
            out_run += popc64(m_gt) + ((eq_next < q ? eq_next : q) - (eq_run < q ? eq_run : q));
            eq_run = eq_next;
        }
    }
}

__global__ __launch_bounds__(kCandThreads) void zero_words_kernel(uint32_t *p, size_t words) {
    const size_t stride = (size_t)gridDim.x * kCandThreads;
    for (size_t i = (size_t)blockIdx.x * kCandThreads + threadIdx.x; i < words; i += stride) p[i] = 0u;
}

template <int VEC, bool DIFF, bool UPDATE>
void launch_collect(const TopkArgs &p, const Ws &w, hipStream_t stream) {
    hipLaunchKernelGGL((split_collect_kernel<VEC, DIFF, UPDATE>), dim3((unsigned)w.G, (unsigned)p.n), dim3(kBlk), 0,
                       stream, p, w);
}

template <bool DIFF, bool UPDATE>
hipError_t launch_select(const TopkArgs &p, const Ws &w, hipStream_t stream) {
    constexpr size_t kDyn = sizeof(uint32_t) * kSelCap;
    static PerDeviceOnce configured;   // per instantiation: the attribute belongs to the function
    const hipError_t cfg = configured([] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&split_select_kernel<DIFF, UPDATE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDyn);
    });
    if (cfg != hipSuccess) return cfg;
    hipLaunchKernelGGL((split_select_kernel<DIFF, UPDATE>), dim3((unsigned)p.n), dim3(kBlk), kDyn, stream, p, w);
    return hipGetLastError();
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
        if (lo < hi) atomicMax(reinterpret_cast<unsigned long long *>(w.hist_a + row * kBinsA), best);
    }
}

template <bool DIFF, bool UPDATE>
__global__ __launch_bounds__(kArgThreads) void argmax_finish_kernel(TopkArgs p, Ws w) {
    const int64_t row = (int64_t)blockIdx.x * kArgThreads + threadIdx.x;
    if (row >= p.n) return;
    unsigned long long *slot = reinterpret_cast<unsigned long long *>(w.hist_a + row * kBinsA);
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
    if (p.k == 1) return launch_argmax(p, w, stream, mk);
    const bool vec4 = (p.d % 4 == 0) && ((uintptr_t)p.a % 16 == 0) && (!diff || (uintptr_t)p.b % 16 == 0);
    if (vec4 && upd) launch_collect<4, true, true>(p, w, stream);
    else if (vec4 && diff) launch_collect<4, true, false>(p, w, stream);
    else if (vec4) launch_collect<4, false, false>(p, w, stream);
    else if (upd) launch_collect<1, true, true>(p, w, stream);
    else if (diff) launch_collect<1, true, false>(p, w, stream);
    else launch_collect<1, false, false>(p, w, stream);
    mk(K_TOPK_COLLECT);
    hipError_t st = hipGetLastError();
    if (st != hipSuccess) return st;

    if (expected_candidates(p.d, p.k) <= (double)kSelectMax) {
        if (upd) st = launch_select<true, true>(p, w, stream);
        else if (diff) st = launch_select<true, false>(p, w, stream);
        else st = launch_select<false, false>(p, w, stream);
        mk(K_TOPK_SELECT);
        return st;
    }
    const dim3 hgrid(kCandBlocks, (unsigned)p.n), hblock(kHistThreads);
    hipLaunchKernelGGL(cand_hist_kernel<1>, hgrid, hblock, 0, stream, p, w);
    mk(K_TOPK_REFINE);
    hipLaunchKernelGGL(cand_hist_kernel<2>, hgrid, hblock, 0, stream, p, w);
    mk(K_TOPK_REFINE);
    const unsigned slot_blocks = (unsigned)((w.nslot + kCandWaves - 1) / kCandWaves);
    const dim3 grid(slot_blocks, (unsigned)p.n), cgrid(slot_blocks + 1, (unsigned)p.n), block(kCandThreads);
    if (upd) hipLaunchKernelGGL((cand_count_kernel<true, true>), cgrid, block, 0, stream, p, w);
    else if (diff) hipLaunchKernelGGL((cand_count_kernel<true, false>), cgrid, block, 0, stream, p, w);
    else hipLaunchKernelGGL((cand_count_kernel<false, false>), cgrid, block, 0, stream, p, w);
    mk(K_TOPK_COUNT);
    if (upd) hipLaunchKernelGGL(cand_emit_kernel<true>, grid, block, 0, stream, p, w);
    else hipLaunchKernelGGL(cand_emit_kernel<false>, grid, block, 0, stream, p, w);
    mk(K_TOPK_EMIT);
    return hipGetLastError();
}

}  // namespace ef21
