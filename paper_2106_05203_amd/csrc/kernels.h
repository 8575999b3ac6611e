// Host-side launchers of the HIP kernels.  Each enqueues on `stream` and returns the HIP status
// of the launch; none of them allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace ef21 {

// Runs `setup` once per HIP device, with that device current: for attributes of a kernel (such as its dynamic LDS
// limit), which the runtime keeps per device.  Thread-safe; a failed setup is tried again by the next call.
struct PerDeviceOnce {
    std::mutex mu;
    bool done[64] = {};
    template <class Setup>
    hipError_t operator()(Setup setup) {
        int dev = 0;
        hipError_t st = hipGetDevice(&dev);
        if (st != hipSuccess) return st;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(mu);
        if (done[dev]) return hipSuccess;
        st = setup();
        if (st == hipSuccess) done[dev] = true;
        return st;
    }
};

// Kernel classes for the optional per-kernel timing of a handle (EF21_K_* in include/ef21.h).
enum KernelId {
    K_GRAD_MAIN = 0,   // the pass(es) over the problem data
    K_GRAD_AUX,        // partial-sum reduction / regulariser
    K_TOPK_ROW,        // one-workgroup-per-row Top-k (+ fused update)
    K_TOPK_COLLECT,    // long rows: the pass over the row that collects candidates
    K_TOPK_SELECT,     // long rows, small k: per-row select + emission on the candidates (+ fused update)
    K_TOPK_REFINE,     // long rows, large k: one digit of the radix select on the candidates
    K_TOPK_COUNT,      // long rows, large k: per-slot counts
    K_TOPK_EMIT,       // long rows, large k: ordered emission (+ fused update)
    K_MODEL_STEP,      // g <- g + mean of the messages and / or x <- x - gamma g
    K_PLUS,            // Algorithm 3: distortions, choice and update of g_i, mean of the rows
    K_SMALL_STEP,      // the whole iteration of Algorithm 2 in one launch (small dense problems)
    K_COUNT
};

// Called after each kernel launch with the class of the kernel just enqueued; a default-constructed
// Marker does nothing.
struct Marker {
    void (*fn)(void *user, int kernel_id) = nullptr;
    void *user = nullptr;
    void operator()(int kernel_id) const {
        if (fn) fn(user, kernel_id);
    }
};

// A dense gradient of eq. (9) left as per-row-block partial sums part[n][chunks][d]: entry (i, j) is
// dense_grad_entry(part + i * chunks * d, chunks, d, j, x[j], m, lambda) (logreg_finish.h).
struct GradParts {
    const float *part = nullptr;
    int64_t chunks = 0;
    int64_t m = 0;
    const float *x = nullptr;
    float lambda = 0.f;
};

// Arguments of one batched Top-k (Section 2.1) over n rows of length d.
//   a, b      v = a - b if b != nullptr (the difference of Algorithm 2, line 5), else v = a
//   out_idx, out_val   [n][k] ascending positions and signed values
//   g_i       if != nullptr (then b must be the same array) the kept entries also update the workers'
//             estimators in place (Algorithm 2, line 6): g_i[row][j] = b[row][j] + v
struct TopkArgs {
    const float *a;
    const float *b;
    int32_t n;
    int64_t d;
    int64_t k;
    int32_t *out_idx;
    float *out_val;
    float *g_i;
    GradParts parts;   // if parts.part != nullptr the rows of `a` are these unreduced gradients (`a` is not read);
                       // launch_topk_row only, d <= 8192, b != nullptr
    int32_t warm;      // launch_topk_split only: 0, or 1 .. 2 = the row thresholds of the last call that named the
                       // same number on this workspace serve as the first guess of this call's (the result never
                       // depends on it; meant for consecutive iterations of one algorithm on one state)
    // launch_topk_split with k > 1 only: if agg_start != nullptr the emission also writes the index that
    // launch_aggregate needs of the messages (aggregate_index_shift), so that its own indexing kernel can be skipped
    int32_t *agg_start;
    int32_t agg_shift;
    int64_t agg_nblk;
};

// One workgroup per row, four radix passes over the row plus an ordered emission.  Needs no
// workspace and is correct for every input; meant for rows that one compute unit can stream
// quickly (and as the reference device path for long rows).
hipError_t launch_topk_row(const TopkArgs &p, hipStream_t stream);

// One workgroup per row that reads the row once and keeps 16 bits of every key in LDS: rows of kRow16Min to
// kRow16Max entries given as they are (p.b == nullptr), k <= kRow16MaxK (meant for rows too long for
// launch_topk_row's LDS copy; the lower limit keeps the kernel's later use of the row copy's LDS, 15 KB of bitmap
// and prefix words, inside the 2 d bytes of the copy).  No workspace.  Other shapes: hipErrorInvalidValue.
constexpr int64_t kRow16Min = 16384, kRow16Max = 61440, kRow16MaxK = 1024;
hipError_t launch_topk_row16(const TopkArgs &p, hipStream_t stream);

// Many workgroups per row for long rows.  Workspace layout and size: topk_split_workspace_bytes.
size_t topk_split_workspace_bytes(int32_t n, int64_t d, int64_t k);
hipError_t launch_topk_split(const TopkArgs &p, void *workspace, hipStream_t stream, const Marker &mk = Marker());
// Two selections of one pass over the same arrays (Algorithm 3, lines 5 to 7): `plain` selects from the rows of a,
// `markov` from a - b (plain.a == markov.a, plain.b == nullptr, same n, d, k >= 2, no g_i update, warm both or
// neither), each with a workspace of its own; norm_parts receives, per row and per piece of the row
// (topk_split_slots(n, d) pieces), the pair (sum a^2, sum (a - b)^2), differences taken exactly and sums in fp64
// in a fixed order: double2 [n][topk_split_slots].
int64_t topk_split_slots(int32_t n, int64_t d);
hipError_t launch_topk_split_pair(const TopkArgs &plain, const TopkArgs &markov, void *ws_plain, void *ws_markov,
                                  void *norm_parts, hipStream_t stream, const Marker &mk = Marker());
// The kernels keep the workspace's histograms and tickets zeroed as long as (n, d) stay the same.
// A workspace that is new, or was last used with another (n, d), needs this reset first.
hipError_t launch_topk_split_reset(void *workspace, int32_t n, int64_t d, hipStream_t stream);

// Algorithm 2, line 3: x <- x - gamma g.
hipError_t launch_model_step(float *x, const float *g, int64_t d, float gamma, hipStream_t stream);

// Algorithm 2, line 8: g <- g + (1/n) sum_i c_i from the messages (idx, val) [n][k] (positions ascending
// and distinct inside a row), summed in worker order, without atomics; if x != nullptr followed, in the
// same pass over the coordinates, by line 3 with the new g.
// `index`: aggregate_index_bytes(n, d) bytes of scratch, overwritten by every call.
// The index: start[w][b] = first pair of worker w's message at or beyond coordinate b << shift, for the blocks
// b = 0 .. nblk of 2^shift coordinates (start[w][nblk] = k), int32 [n][nblk + 1].  aggregate_index_shift gives the
// shift that launch_aggregate uses for a shape (nblk = ceil(d / 2^shift)), or -1 if it uses no index for it.
// index_ready: the caller has already written the index (launch_topk_split can); otherwise a kernel of the call does.
size_t aggregate_index_bytes(int32_t n, int64_t d);
int aggregate_index_shift(int32_t n, int64_t k, int64_t d);
hipError_t launch_aggregate(const int32_t *idx, const float *val, int32_t n, int64_t k, int64_t d, float *g, float *x,
                            float gamma, void *index, hipStream_t stream, bool index_ready = false);

// g = (1/n) sum_i g_i (input line of Algorithm 2), summed in worker order.
hipError_t launch_mean_rows(const float *g_i, float *g, int32_t n, int64_t d, hipStream_t stream);

// `loss` below: the per-row loss of the linear model (LossKind in device_utils.h): logistic (eq. (9)) or squared.
// kLossHalfSquare (z^2 / 2, no target) is internal: its gradient is (1/m) A_i^T A_i x, the product the power
// iteration needs.  x_stride below: 0 = one x [d] for all workers, d = a row of x [n][d] per worker.
enum { kLossLogistic = 0, kLossLeastSquares = 1, kLossHalfSquare = 2 };

// The minibatch of Algorithm 5: worker i's gradient estimator sums the rows rows[i][0..tau) of its m rows
// (tau <= m; an entry outside [0, m) contributes nothing) and divides by tau.  tau == 0: all rows, the gradient.
struct RowBatch {
    const int32_t *rows = nullptr;   // device, [n][tau]
    int64_t tau = 0;
};

// Gradient of eq. (9) for all workers, dense rows.  scratch: logreg_dense_scratch_bytes.  With defer != nullptr
// the last reduction may be left to the consumer: then *defer describes the partial sums (they live in
// scratch until the next call) and grad is not written; defer->part == nullptr means grad was written.
size_t logreg_dense_scratch_bytes(int32_t n, int64_t m, int64_t d);
hipError_t launch_logreg_grad_dense(const float *A, const float *y, const float *x, float *grad, int32_t n,
                                    int64_t m, int64_t d, float lambda, void *scratch, hipStream_t stream,
                                    const Marker &mk = Marker(), GradParts *defer = nullptr,
                                    int loss = kLossLogistic, RowBatch batch = RowBatch(), int64_t x_stride = 0);

// Gradient of eq. (9) for all workers, CSR rows with nnz entries in all.  `index`
// (logreg_csr_index_bytes bytes, owned by the caller) is built once per problem by logreg_csr_build_index
// and holds per-row column-range offsets, a range-major and a column-major copy of the matrix (6 bytes per
// entry each) and scratch for the two-pass kernels.  The build synchronises the stream and reports whether those
// kernels can be used (every row's columns ascending and inside [0, d), fewer than 2^31 entries per
// worker); pass index = nullptr to launch_logreg_grad_csr otherwise.  Under a row batch the work is
// proportional to the batch: one wavefront per listed row and global fp32 atomics, whatever the index.
size_t logreg_csr_index_bytes(int32_t n, int64_t m, int64_t d, int64_t nnz);
hipError_t logreg_csr_build_index(const int64_t *rowptr, const int32_t *col, const float *val, int32_t n, int64_t m,
                                  int64_t d, int64_t nnz, void *index, hipStream_t stream, bool *usable);
hipError_t launch_logreg_grad_csr(const int64_t *rowptr, const int32_t *col, const float *val, const float *y,
                                  const float *x, float *grad, int32_t n, int64_t m, int64_t d, int64_t nnz,
                                  float lambda, const void *index, hipStream_t stream, const Marker &mk = Marker(),
                                  int loss = kLossLogistic, RowBatch batch = RowBatch(), int64_t x_stride = 0);

// Small dense problems: lines 5, 6, 8 (and 3 if take_step) of Algorithm 2 in ONE launch, from the problem and the
// state, with the arithmetic of the separate kernels (gradient, row Top-k with update, aggregation), so the
// results are the same bits.  small_step_applies says whether the shape qualifies (d <= 1024, n * k <= 2048,
// n * m * d <= 2^24, ...).  scratch: logreg_dense_scratch_bytes; tickets: small_step_ticket_bytes(n) bytes,
// zero before the first launch (the kernel leaves them zero).
bool small_step_applies(const float *A, int32_t n, int64_t m, int64_t d, int64_t k);
size_t small_step_ticket_bytes(int32_t n);
hipError_t launch_small_step(const float *A, const float *y, float *x, float *g, float *g_i, int32_t n, int64_t m,
                             int64_t d, int64_t k, float lambda, float gamma, int loss, bool take_step, void *scratch,
                             void *tickets, int32_t *msg_idx, float *msg_val, hipStream_t stream);

// Algorithm 3 (EF21+), lines 7 and 8, for all workers: from the gradients s [n][d], the estimators g_i [n][d]
// (updated in place) and the two Top-k results (idx_b, val_b) = C(s), (idx_m, val_m) = C(s - g_i), all [n][k]:
// BM[i] = (B_i, M_i), branch[i] = 1 where the plain compressor wins (M_i > B_i), (msg_idx, msg_val) = the chosen
// pairs, and g_i <- b or m accordingly.  scratch: plus_scratch_bytes(n, d, k) bytes.  If norm_chunks > 0 the
// leading double2 [n][norm_chunks] of scratch already hold partial sums of (s^2, (s - g_i)^2) per row (from
// launch_topk_split_pair; norm_chunks <= plus_norm_chunks_max(n, d)) and the pass over s and g_i is skipped.
size_t plus_scratch_bytes(int32_t n, int64_t d, int64_t k);
int64_t plus_norm_chunks_max(int32_t n, int64_t d);
hipError_t launch_plus_choose(const float *s, float *g_i, int32_t n, int64_t d, int64_t k, const int32_t *idx_b,
                              const float *val_b, const int32_t *idx_m, const float *val_m, void *scratch,
                              int32_t *branch, double *BM, int32_t *msg_idx, float *msg_val, hipStream_t stream,
                              int64_t norm_chunks = 0);

// Power iteration for the smoothness constants of Section 3.4: v [rows][d] <- a fixed positive start vector;
// and one step: stats[row] = (v^T w / v^T v, |w| / |v|) as two doubles, v <- w / |w|, for w = M v, M symmetric
// positive semidefinite (both numbers are lower bounds of its largest eigenvalue).
hipError_t launch_power_start(float *v, int32_t rows, int64_t d, hipStream_t stream);
hipError_t launch_power_step(const float *w, float *v, int32_t rows, int64_t d, double *stats, hipStream_t stream);

// Algorithm 4 (EF): e <- e + gamma s over all n * d entries; e <- 0 at the kept positions idx [n][k]; v <- 0.
hipError_t launch_ef_accumulate(const float *s, float *e, int32_t n, int64_t d, float gamma, hipStream_t stream);
hipError_t launch_ef_clear_kept(const int32_t *idx, int32_t n, int64_t k, float *e, int64_t d, hipStream_t stream);
hipError_t launch_fill_zero(float *v, int64_t d, hipStream_t stream);

// Plain streaming kernels for measuring what the HBM delivers: one read of `n16` 16-byte words (their sum goes
// to sink[0]), and a copy.
hipError_t launch_hbm_read(const void *src, int64_t n16, float *sink, hipStream_t stream);
hipError_t launch_hbm_copy(void *dst, const void *src, int64_t n16, hipStream_t stream);

}  // namespace ef21
