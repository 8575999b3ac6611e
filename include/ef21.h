/*
 * libef21 -- the data-parallel hot path of EF21 (Richtarik, Sokolov, Fatkhullin,
 * arXiv 2106.05203) on one AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * The library solves the paper's problem  min_x f(x) = (1/n) sum_i f_i(x)  (eq. (1)) with
 * Algorithm 2 ("EF21, multiple nodes"), all n workers batched as rows on one GPU:
 *
 *     line 3   x   <- x - gamma * g
 *     line 5   c_i  = C(grad f_i(x) - g_i)          C = Top-k (Section 2.1)
 *     line 6   g_i <- g_i + c_i
 *     line 8   g   <- g + (1/n) sum_i c_i
 *
 * Conventions that hold for every call
 *   - Every array argument is a DEVICE pointer to memory the caller owns (for example the
 *     storage of a PyTorch tensor), row-major and contiguous.  Values are fp32, indices are
 *     int32, sizes are int64.  The library copies what it needs to keep (state); it only
 *     borrows problem data (see ef21_set_problem_*).
 *   - Work is enqueued on a HIP stream and the call returns without waiting for it.  The
 *     caller synchronises the stream before reading results on the host.
 *   - Every function except ef21_create and ef21_last_error returns an EF21_* status.  On
 *     failure nothing has been enqueued unless stated, and ef21_last_error() describes it.
 *   - NaN inputs are outside the contract: a NaN ranks above +inf in Top-k (its bit pattern
 *     is larger); nothing traps.
 *   - A handle is not thread safe; different handles may be used from different threads.
 */
#ifndef EF21_H
#define EF21_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ef21_ctx *ef21_handle;

enum {
    EF21_OK = 0,
    EF21_EINVAL = -1, /* bad argument (size, NULL pointer, gamma)                       */
    EF21_ENOMEM = -2, /* device or host allocation failed                                */
    EF21_EHIP = -3,   /* a HIP runtime call failed; text in ef21_last_error()            */
    EF21_ESTATE = -4  /* call not possible in the handle's state (e.g. no problem set)   */
};

/* flags of ef21_step (one order, optionally or-ed with EF21_PLUS or EF21_ONE_LAUNCH) */
enum {
    EF21_ORDER_GRAD_FIRST = 0u, /* lines 5, 6, 8 at the current x, then line 3 (default)      */
    EF21_ORDER_STEP_FIRST = 1u, /* line 3, then lines 5, 6, 8 at the new x (loop as printed)  */
    EF21_PLUS = 2u,             /* the loop body of Algorithm 3 (EF21+) instead of Algorithm 2 */
    EF21_CLASSIC_EF = 4u,       /* one round of Algorithm 4 (the original EF); no order, no EF21_PLUS */
    EF21_ONE_LAUNCH = 8u        /* the whole pass as one kernel where the problem qualifies (see ef21_step) */
};

/* Human-readable text of the calling thread's last failure ("" if none).  Library-owned. */
const char *ef21_last_error(void);

/*
 * Input line of Algorithm 2: n workers, dimension d, Top-k parameter k (1 <= k <= d), learning
 * rate gamma > 0 (finite).  Allocates, on the current HIP device, the state x [d], g [d],
 * g_i [n][d] (all zero) and the last messages (idx, val) [n][k].  Returns NULL on failure.
 * d must be below 2^31 (indices are int32) and n at most 65535 (a worker is a row of the launch grids).
 */
ef21_handle ef21_create(int32_t n, int64_t d, int64_t k, float gamma);

/* Waits for the handle's stream, then frees everything the handle owns.  NULL is allowed. */
int ef21_destroy(ef21_handle h);

/* Stream (a hipStream_t passed as void*) that later calls on this handle enqueue on.  The
 * stream is borrowed.  Default: the null stream. */
int ef21_set_stream(ef21_handle h, void *hip_stream);

/*
 * Top-k compressor of Section 2.1, batched over rows, stateless:  for each of the n rows of
 * `rows` [n][d] keep the k entries of largest absolute value.  Magnitudes are compared as
 * the fp32 bit pattern with the sign bit cleared, so +a ties with -a and +0 with -0; among
 * equal magnitudes the LOWER index is kept (the paper does not specify ties).
 *   out_idx [n][k]  kept positions of each row in ASCENDING order
 *   out_val [n][k]  the (signed) input values at those positions
 * Exactly k pairs are produced per row even if fewer than k entries are non-zero.
 * Enqueued on `hip_stream` (NULL = null stream).  For rows longer than a few 10^4 entries the
 * call uses a device workspace (about 8 d + 90 000 bytes per row) that the library keeps per device and
 * stream and grows on demand with hipMalloc (a growing call waits for that stream first).  Calls on
 * different streams use different workspaces and may overlap; calls on one stream run one after the other.
 * The workspaces are kept until the process ends (a device that has seen more than 16 streams frees all
 * of its workspaces after a device-wide wait and starts over).  ef21_topk_static never allocates.
 * EF21_EINVAL: n < 1, n > 65535 (a row is a row of the launch grids), d < 1, d >= 2^31, k < 1, k > d, NULL pointer.
 */
int ef21_topk(const float *rows, int32_t n, int64_t d, int64_t k, int32_t *out_idx, float *out_val,
              void *hip_stream);

/*
 * ef21_topk for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results (the same kernels) as ef21_topk, but the workspace
 * of the long-row path is a 64 MiB array that is part of the library's device image (each GPU the library runs on
 * holds it until the process ends), so the call allocates nothing, frees nothing and synchronises nothing: it
 * enqueues kernels on `hip_stream` and returns.  Rows of 16384 entries or more that are not selected by one
 * workgroup per row (d > 61440 or k > 1024) need about 8 d + 90 000 bytes of workspace per row; a call whose
 * n rows need more than the 64 MiB (for example more than eight rows of 10^6 entries) is rejected with EF21_EINVAL
 * and a message that gives both sizes -- use ef21_topk for those.  Shorter rows need no workspace and have no limit.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads) race and
 * give wrong results; calls that follow one another on a stream, of any shapes, are fine (each call clears the
 * part of the array that must start at zero with a fill kernel of its own, so it may also be captured into a graph).
 * Errors otherwise as ef21_topk.
 */
int ef21_topk_static(const float *rows, int32_t n, int64_t d, int64_t k, int32_t *out_idx, float *out_val,
                     void *hip_stream);

/*
 * Attach the objective of Section 5, eq. (9): logistic loss with the non-convex regulariser,
 *   f_i(x) = (1/m) sum_l log(1 + exp(-y_il a_il^T x)) + lambda sum_j x_j^2 / (1 + x_j^2),
 * each worker holding m rows (each f_i carries the full regulariser, so (1/n) sum_i f_i is
 * eq. (9) for an even split of the data).
 *   dense:  A [n][m][d] fp32, y [n][m] fp32 in {-1, +1}
 *   csr:    one CSR over all n*m rows, worker i owning rows i*m .. (i+1)*m-1:
 *           rowptr [n*m+1] int64, col [nnz] int32 in [0, d), val [nnz] fp32, y [n][m]
 * The arrays are BORROWED: they must stay valid and unchanged while the handle uses them.
 * Allocates a gradient buffer [n][d] and scratch on first use.  The csr call also reads the matrix
 * once (it waits for the stream): if every row's columns are strictly ascending and inside [0, d),
 * and no worker holds 2^31 - 2^16 entries or more, it builds what the fast two-pass gradient kernels
 * need -- a small per-row index of column ranges and two re-ordered copies of the matrix with 16-bit
 * indices (about 12 bytes per entry plus 4 n (d + 1) + 4 (n m + n) ceil(d / 12288) bytes of device
 * memory in all, owned by the handle).  Otherwise a slower kernel based on global floating-point
 * atomics is used, in which columns outside [0, d) are skipped.
 */
int ef21_set_problem_dense(ef21_handle h, const float *A, const float *y, int64_t m, float lambda);
int ef21_set_problem_csr(ef21_handle h, const int64_t *rowptr, const int32_t *col, const float *val,
                         const float *y, int64_t m, float lambda);

/*
 * The per-row loss of the attached problem (default EF21_LOSS_LOGISTIC).  With EF21_LOSS_LEAST_SQUARES the
 * objective is the one of Section 5.2,
 *   f_i(x) = (1/m) sum_l (a_il^T x - y_il)^2  (+ the regulariser of eq. (9) times lambda; pass lambda = 0 for
 *   the paper's function), y holding the targets b_il,
 * whose gradient is (2/m) sum_l (a_il^T x - y_il) a_il: the same kernels with another derivative per row.
 * Takes effect from the next gradient.  EF21_EINVAL: unknown value.
 */
enum { EF21_LOSS_LOGISTIC = 0, EF21_LOSS_LEAST_SQUARES = 1 };
int ef21_set_loss(ef21_handle h, int loss);

/*
 * Stochastic gradients (Algorithm 5, the extension of Algorithm 2 in the appendix): from the next gradient
 * on, worker i's gradient is replaced by the minibatch estimator
 *   ghat_i = (1/tau) sum over l in rows[i][0..tau) of the gradient of row l's loss  +  the regulariser's,
 * in ef21_local_grad and in every variant of ef21_step.  rows: device, int32 [n][tau], row numbers inside
 * the worker's m rows, drawn by the caller (the library draws no random numbers); borrowed and read at
 * every gradient, so the caller redraws a batch by rewriting the buffer (stream-ordered) or by another call.
 * A row listed twice counts twice; an entry outside [0, m) contributes nothing and is never dereferenced
 * (the division stays by tau).  tau == 0 (rows ignored): back to the full gradient.  Attaching a problem
 * resets it.  Dense rows run the ordinary kernels over the listed rows (bitwise reproducible); CSR rows take
 * one wavefront per listed row and global fp32 atomics (reproducible to rounding), work proportional to
 * the batch.  EF21_ESTATE without a problem; EF21_EINVAL: tau outside [0, m], or rows NULL with tau > 0.
 */
int ef21_set_minibatch(ef21_handle h, const int32_t *rows, int64_t tau);

/*
 * The largest stepsize Theorem 1 allows for the attached problem (Section 3.4, the bound on gamma in the theorem),
 *   gamma = 1 / (L + Ltilde sqrt(beta / theta)),   sqrt(beta / theta) = (1 + sqrt(1 - alpha)) / alpha - 1,
 * alpha = k / d for Top-k, Ltilde the quadratic mean of the workers' smoothness constants
 *   L_i = c lambda_max((1/m) A_i^T A_i) + 2 lambda
 * (c = 1/4 for the logistic loss, 2 for least squares: the largest curvature of the per-row loss; 2 is the
 * largest curvature of t^2 / (1 + t^2)), and L = c lambda_max((1/(n m)) sum_i A_i^T A_i) + 2 lambda for f itself.
 * The eigenvalues come from `iterations` steps of the power iteration on the GPU (each step two passes of
 * the gradient kernels over the problem), started from a fixed positive vector; the estimate |M v| for the
 * unit vector v of the last step approaches lambda_max from below, so few iterations give a stepsize that is
 * too large by the same factor: 100 to 300 steps bring problems without a dominant direction within about one
 * per cent.  gamma, L, L_i [n]: host memory, each may be NULL.  Uses the handle's loss, lambda and k, and all
 * rows whatever ef21_set_minibatch says; the handle's stepsize is not changed.  The first call on a handle
 * allocates (n + 2) d floats that the handle keeps; every call overwrites the handle's gradient buffer and
 * returns after the stream has drained.
 * EF21_ESTATE without a problem; EF21_EINVAL: iterations outside [1, 10^6]; EF21_ENOMEM.
 */
int ef21_theory_stepsize(ef21_handle h, int32_t iterations, double *gamma, double *L, double *L_i);

/*
 * State of Algorithm 2.  set: copies x [d] and g_i [n][d] into the handle (either may be NULL
 * = keep); g [d] NULL means "recompute g = (1/n) sum_i g_i" (the algorithm's input line).
 * get: copies the handle's state out; any pointer may be NULL.
 */
int ef21_set_state(ef21_handle h, const float *x, const float *g_i, const float *g);
int ef21_get_state(ef21_handle h, float *x, float *g_i, float *g);

/* The messages c_i of the last ef21_step as (idx, val) [n][k], layout as in ef21_topk. */
int ef21_get_messages(ef21_handle h, int32_t *idx, float *val);

/*
 * grad f_i(x) for all workers (derivative of eq. (9)):
 *   (1/m) sum_l  -y_il / (1 + exp(y_il a_il^T x)) a_il  +  2 lambda x_j / (1 + x_j^2)^2
 * at `x` [d] (NULL = the handle's x), written to out_grad [n][d].  EF21_ESTATE without a
 * problem.  fp32 arithmetic; sums over rows are taken in a fixed order (bitwise reproducible),
 * except in the atomics-based kernel for CSR rows with unsorted columns (reproducible to rounding).
 */
int ef21_local_grad(ef21_handle h, const float *x, float *out_grad);

/*
 * One pass of the loop body of Algorithm 2 for all workers.
 *   grads [n][d]: the vectors used in place of grad f_i(x) in line 5 (supplied gradients,
 *   e.g. the stochastic estimators of Algorithm 5), or NULL to compute grad f_i at the
 *   handle's x from the attached problem (EF21_ESTATE if none).
 *   flags: EF21_ORDER_GRAD_FIRST or EF21_ORDER_STEP_FIRST.  With supplied gradients and
 *   STEP_FIRST the caller must have evaluated them at x - gamma*g.
 * The difference in line 5 is one fp32 subtraction; line 6 is one fp32 addition per kept
 * entry; line 8 adds the messages per coordinate in worker order in fp32 and applies
 * g + sum * (1/n) as one fused multiply-add; line 3 is one fused multiply-add per coordinate.
 * With supplied gradients every result (messages, g_i, g, x) is bitwise reproducible.
 * With EF21_ONE_LAUNCH in flags, a small dense problem (grads NULL, d <= 1024, n * k <= 2048,
 * n * m * d <= 2^24, no minibatch, no EF21_PLUS) runs the whole pass as ONE kernel: the same arithmetic in the
 * same order as the separate gradient, Top-k and aggregation kernels, so the results are the same bits.  It
 * saves two launches and pays for them in device-scope fences: measured on par with the separate kernels for
 * a handful of workers and slower for twenty, hence not the default.  Where the problem does not qualify the
 * flag changes nothing.
 * EF21_EINVAL: unknown flag bits, or EF21_CLASSIC_EF together with an order or EF21_PLUS.
 */
int ef21_step(ef21_handle h, const float *grads, uint32_t flags);

/*
 * With EF21_PLUS in flags, ef21_step runs the loop body of Algorithm 3 (EF21+, Section 3.5) on the same
 * state: with s = grad f_i(x) (or the supplied row) every worker forms b = C(s) (line 5) and
 * m = g_i + C(s - g_i) (line 6), C = Top-k as in ef21_topk; the distortions B = ||b - s||^2 and
 * M = ||m - s||^2 (line 7) are computed in fp64 as ||s||^2 and ||s - g_i||^2 minus the sums of the kept
 * squares, every sum in a fixed order; g_i <- m if M <= B, else b (line 8); g <- (1/n) sum_i g_i, the
 * rows added in worker order in fp64 and the mean rounded once (line 10).  ef21_get_messages then returns, per worker, the k pairs
 * of the compressor it chose.  The first such call on a handle allocates (and waits for the stream).
 *
 * ef21_get_choices copies out what the last EF21_PLUS step decided: branch [n] int32 (1 = the plain
 * compressor b was chosen, 0 = the Markov compressor m) and distortions [n][2] fp64 (B_i, M_i); either
 * pointer may be NULL.  EF21_ESTATE before the first EF21_PLUS step.
 */
int ef21_get_choices(ef21_handle h, int32_t *branch, double *distortions);

/*
 * With flags == EF21_CLASSIC_EF, ef21_step runs one round of Algorithm 4 (EF, the original error feedback
 * that Section 4 compares EF21 with) on the same handle, the workers' errors e_i taking the place of g_i in
 * ef21_set_state / ef21_get_state (start from e_i = 0): at the handle's x, with s = grad f_i(x) or the
 * supplied row,  p_i = e_i + gamma s  (one fused multiply-add per entry, written over e_i),
 * w_i = C(p_i)  (Top-k as in ef21_topk; returned by ef21_get_messages),  e_i = p_i - w_i  (zero at the kept
 * positions),  x <- x - (1/n) sum_i w_i  (the sum per coordinate in worker order in fp32).  Started from
 * e_i = 0 this produces the iterates x^0, x^1, ... of Algorithm 4.  The g of ef21_get_state holds
 * (1/n) sum_i w_i of the last round.  Do not mix rounds of different algorithms on one state.
 */

/*
 * Per-kernel timing, for measurement only (not part of the paper's method).  While enabled,
 * ef21_step and ef21_local_grad record one HIP event on the handle's stream after each kernel
 * they launch; the time between consecutive events is charged to the class of the later kernel.
 * ef21_set_timing and ef21_get_timing wait for the stream.  ms[EF21_K_COUNT] receives the
 * accumulated milliseconds per class and launches[EF21_K_COUNT] the number of intervals (either
 * may be NULL); reset != 0 clears the sums.  Classes, in order (names from ef21_kernel_name):
 * grad_main, grad_aux, topk_row, topk_collect, topk_select, topk_refine, topk_count, topk_emit,
 * model_step, plus (what is particular to Algorithm 3), small_step (the one-launch iteration).
 */
enum { EF21_K_COUNT = 11 };
int ef21_set_timing(ef21_handle h, int enabled);
int ef21_get_timing(ef21_handle h, double *ms, int64_t *launches, int reset);
const char *ef21_kernel_name(int kernel_class);

/*
 * Plain streaming kernels, for measurement only (not part of the paper's method): what this GPU's HBM
 * delivers to the simplest possible kernel, to set beside the vendor's peak.  Both take DEVICE pointers to
 * 16-byte aligned buffers of `bytes` bytes (a multiple of 16) and enqueue one kernel on `hip_stream`.
 *   ef21_hbm_read   reads `src` once with the same non-temporal loads the library's kernels use and
 *                   writes one float to sink[0] (sink may alias nothing else)
 *   ef21_hbm_copy   dst <- src
 * EF21_EINVAL: NULL pointer, misaligned pointer, bytes < 16 or not a multiple of 16.
 */
int ef21_hbm_read(const void *src, int64_t bytes, float *sink, void *hip_stream);
int ef21_hbm_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EF21_H */
