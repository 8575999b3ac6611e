// C ABI of libef21 (declared in include/ef21.h): argument checks, the handle, launches.
#include <cmath>
#include <cstdio>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/ef21.h"
#include "kernels.h"

// Workspace of ef21_topk_static: device memory that exists from the moment the library is loaded, so that call
// never allocates.  Every GPU holds its own copy at its own address; host code reaches it only through the address
// that hipGetSymbolAddress returns with that GPU current, never through the array's name.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string &msg) {
    g_last_error = msg;
    return code;
}

int fail_hip(hipError_t st, const char *what) {
    return fail(EF21_EHIP, std::string(what) + ": " + hipGetErrorString(st));
}

#define EF21_HIP(call)                                           \
    do {                                                         \
        hipError_t st__ = (call);                                \
        if (st__ != hipSuccess) return fail_hip(st__, #call);    \
    } while (0)

static_assert((int)ef21::K_COUNT == (int)EF21_K_COUNT, "kernel classes of kernels.h and ef21.h must agree");

enum ProblemKind { kNone = 0, kDense = 1, kCSR = 2 };

// Rows at least this long are selected with many workgroups per row.
constexpr int64_t kSplitMinRow = 1 << 14;

bool use_split(int64_t d) { return d >= kSplitMinRow; }

// Workspaces of the stateless ef21_topk: one per (device, stream), so that calls on different streams never share
// one (calls on one stream run one after the other).  They live until the process ends; if a device collects more
// than kMaxTopkStreams of them, all of that device's are freed after a device-wide wait and the list starts over.
struct StreamWorkspace {
    int device = -1;
    hipStream_t stream = nullptr;
    void *ptr = nullptr;
    size_t bytes = 0;
    int32_t last_n = 0;           // shape of the last call: the layout inside the workspace depends on it
    int64_t last_d = 0;
};
constexpr size_t kMaxTopkStreams = 16;
struct SharedWorkspaces {
    std::mutex mu;
    std::vector<StreamWorkspace> list;
};
SharedWorkspaces g_topk_ws;

// Per-device address of `scratch`.
struct StaticScratch {
    std::mutex mu;
    void *ptr[64] = {};           // per device, looked up on the first call with that device current
};
StaticScratch g_static_ws;

// Rows that the long-row path selects with a workspace (the others are selected by one workgroup each, without).
bool topk_needs_workspace(int64_t d, int64_t k) {
    return use_split(d) && !(d <= ef21::kRow16Max && k <= ef21::kRow16MaxK);
}

}  // namespace

// Optional per-kernel timing of a handle: one HIP event after every kernel launch of ef21_step /
// ef21_local_grad; the time between consecutive events is charged to the later kernel's class.
struct Timing {
    struct Rec {
        int kernel;          // -1 marks the start of a call
        hipEvent_t ev;
    };
    bool on = false;
    std::vector<hipEvent_t> pool;
    std::vector<Rec> recs;
    double ms[ef21::K_COUNT] = {};
    int64_t launches[ef21::K_COUNT] = {};
};

struct ef21_ctx {
    int32_t n = 0;
    int64_t d = 0, k = 0;
    float gamma = 0.f;
    int device = 0;
    hipStream_t stream = nullptr;
    // state of Algorithm 2
    float *x = nullptr, *g = nullptr, *g_i = nullptr;
    int32_t *msg_idx = nullptr;
    float *msg_val = nullptr;
    // problem (borrowed)
    ProblemKind kind = kNone;
    const float *A = nullptr, *y = nullptr, *val = nullptr;
    const int64_t *rowptr = nullptr;
    const int32_t *col = nullptr;
    int64_t m = 0;
    float lambda = 0.f;
    int loss = 0;                   // EF21_LOSS_*
    ef21::RowBatch batch;           // Algorithm 5 (borrowed); tau == 0: full gradients
    // owned buffers for the problem path and the long-row Top-k
    float *grad = nullptr;
    void *scratch = nullptr;
    size_t scratch_bytes = 0;
    void *topk_ws = nullptr;
    void *topk_ws2 = nullptr;       // second long-row workspace: the plain compressor of Algorithm 3
    void *agg_index = nullptr;      // runs of the messages per coordinate sub-block (scratch of line 8)
    void *tickets = nullptr;        // counters of the one-launch iteration (zero between launches)
    void *csr_index = nullptr;      // column-range index of the attached CSR problem
    bool csr_indexed = false;
    int64_t nnz = 0;                // entries of the attached CSR problem
    // Algorithm 3 (allocated by the first EF21_PLUS step)
    int32_t *plus_idx = nullptr;    // [2][n][k]: C(s), then C(s - g_i)
    float *plus_val = nullptr;
    void *plus_scratch = nullptr;
    int32_t *plus_branch = nullptr; // [n]
    double *plus_bm = nullptr;      // [n][2]
    // power iteration of ef21_theory_stepsize (allocated by the first call)
    float *power_v = nullptr;       // [n + 2][d]
    double *power_stats = nullptr;  // [n + 1][2]
    Timing timing;
};

namespace {

int check_handle(ef21_handle h) {
    if (!h) return fail(EF21_EINVAL, "handle is NULL");
    int dev = -1;
    EF21_HIP(hipGetDevice(&dev));
    if (dev != h->device) return fail(EF21_ESTATE, "the handle was created on another HIP device than the current one");
    return EF21_OK;
}

int check_topk_sizes(int32_t n, int64_t d, int64_t k) {
    if (n < 1 || n > 65535) return fail(EF21_EINVAL, "n must be in [1, 65535]");
    if (d < 1 || d >= ((int64_t)1 << 31)) return fail(EF21_EINVAL, "d must be in [1, 2^31)");
    if (k < 1 || k > d) return fail(EF21_EINVAL, "k must be in [1, d]");
    return EF21_OK;
}

void record_mark(void *user, int kernel_id) {
    ef21_ctx *c = (ef21_ctx *)user;
    Timing &t = c->timing;
    if (!t.on) return;
    hipEvent_t ev = nullptr;
    if (!t.pool.empty()) {
        ev = t.pool.back();
        t.pool.pop_back();
    } else if (hipEventCreate(&ev) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    (void)hipEventRecord(ev, c->stream);
    t.recs.push_back({kernel_id, ev});
}

ef21::Marker marker_of(ef21_ctx *c) {
    ef21::Marker m;
    if (c->timing.on) {
        m.fn = record_mark;
        m.user = c;
    }
    return m;
}

// Folds the recorded events into the per-class sums.  The stream must be idle.
void drain_timing(ef21_ctx *c) {
    Timing &t = c->timing;
    for (size_t i = 0; i < t.recs.size(); ++i) {
        if (i > 0 && t.recs[i].kernel >= 0) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, t.recs[i - 1].ev, t.recs[i].ev) == hipSuccess) {
                t.ms[t.recs[i].kernel] += ms;
                t.launches[t.recs[i].kernel] += 1;
            } else {
                (void)hipGetLastError();
            }
        }
    }
    for (auto &r : t.recs) t.pool.push_back(r.ev);
    t.recs.clear();
}

void free_ctx(ef21_ctx *c) {
    if (!c) return;
    for (auto &r : c->timing.recs) (void)hipEventDestroy(r.ev);
    for (auto ev : c->timing.pool) (void)hipEventDestroy(ev);
    (void)hipFree(c->x);
    (void)hipFree(c->g);
    (void)hipFree(c->g_i);
    (void)hipFree(c->msg_idx);
    (void)hipFree(c->msg_val);
    (void)hipFree(c->grad);
    (void)hipFree(c->scratch);
    (void)hipFree(c->topk_ws);
    (void)hipFree(c->topk_ws2);
    (void)hipFree(c->csr_index);
    (void)hipFree(c->agg_index);
    (void)hipFree(c->tickets);
    (void)hipFree(c->plus_idx);
    (void)hipFree(c->plus_val);
    (void)hipFree(c->plus_scratch);
    (void)hipFree(c->plus_branch);
    (void)hipFree(c->plus_bm);
    (void)hipFree(c->power_v);
    (void)hipFree(c->power_stats);
    delete c;
}

int ensure_problem_buffers(ef21_ctx *c, size_t scratch_bytes) {
    if (!c->grad) {
        hipError_t st = hipMalloc((void **)&c->grad, sizeof(float) * (size_t)c->n * c->d);
        if (st != hipSuccess) return fail(EF21_ENOMEM, "hipMalloc of the gradient buffer failed");
    }
    if (scratch_bytes > c->scratch_bytes) {
        EF21_HIP(hipStreamSynchronize(c->stream));
        (void)hipFree(c->scratch);
        c->scratch = nullptr;
        c->scratch_bytes = 0;
        hipError_t st = hipMalloc(&c->scratch, scratch_bytes);
        if (st != hipSuccess) return fail(EF21_ENOMEM, "hipMalloc of the gradient scratch failed");
        c->scratch_bytes = scratch_bytes;
    }
    return EF21_OK;
}

// defer != nullptr: the dense gradient may stay in partial sums for the row Top-k kernel to finish.
int enqueue_local_grad(ef21_ctx *c, const float *x, float *out, ef21::GradParts *defer = nullptr) {
    hipError_t st;
    const ef21::Marker mk = marker_of(c);
    if (defer) *defer = ef21::GradParts();
    if (c->kind == kDense)
        st = ef21::launch_logreg_grad_dense(c->A, c->y, x, out, c->n, c->m, c->d, c->lambda, c->scratch, c->stream,
                                            mk, defer, c->loss, c->batch);
    else
        st = ef21::launch_logreg_grad_csr(c->rowptr, c->col, c->val, c->y, x, out, c->n, c->m, c->d, c->nnz,
                                          c->lambda, c->csr_indexed ? c->csr_index : nullptr, c->stream, mk, c->loss,
                                          c->batch);
    if (st != hipSuccess) return fail_hip(st, "gradient kernel launch");
    return EF21_OK;
}

// index_ready (may be nullptr): the message index of the aggregation, asked for through p.agg_start, was written.
int enqueue_topk(ef21::TopkArgs p, void *workspace, hipStream_t stream, const ef21::Marker &mk,
                 bool *index_ready = nullptr) {
    hipError_t st;
    const bool split = use_split(p.d) && workspace && !(p.d <= ef21::kRow16Max && p.k <= ef21::kRow16MaxK && !p.b && !p.parts.part);
    if (!(split && p.k > 1)) p.agg_start = nullptr;
    if (index_ready) *index_ready = p.agg_start != nullptr;
    if (use_split(p.d) && p.d <= ef21::kRow16Max && p.k <= ef21::kRow16MaxK && !p.b && !p.parts.part) {
        st = ef21::launch_topk_row16(p, stream);
        mk(ef21::K_TOPK_ROW);
    } else if (use_split(p.d) && workspace) {
        st = ef21::launch_topk_split(p, workspace, stream, mk);
    } else {
        st = ef21::launch_topk_row(p, stream);
        mk(ef21::K_TOPK_ROW);
    }
    if (st != hipSuccess) return fail_hip(st, "Top-k kernel launch");
    return EF21_OK;
}

// Asks the Top-k (long rows only) to write the index of the messages that launch_aggregate would otherwise build.
void want_message_index(const ef21_ctx *c, ef21::TopkArgs *p) {
    const int shift = ef21::aggregate_index_shift(c->n, c->k, c->d);
    if (shift < 0) return;
    p->agg_start = (int32_t *)c->agg_index;
    p->agg_shift = shift;
    p->agg_nblk = ((c->d - 1) >> shift) + 1;
}

// The long-row workspace of a handle keeps one layout for life: zero its control part once.
hipError_t alloc_split_workspace(void **ptr, size_t bytes, int32_t n, int64_t d) {
    hipError_t st = hipMalloc(ptr, bytes);
    if (st != hipSuccess) return st;
    st = ef21::launch_topk_split_reset(*ptr, n, d, nullptr);
    if (st == hipSuccess) st = hipDeviceSynchronize();
    if (st != hipSuccess) {
        (void)hipFree(*ptr);
        *ptr = nullptr;
    }
    return st;
}

}  // namespace

extern "C" {

const char *ef21_last_error(void) { return g_last_error.c_str(); }

ef21_handle ef21_create(int32_t n, int64_t d, int64_t k, float gamma) {
    if (check_topk_sizes(n, d, k) != EF21_OK) return nullptr;
    if (!(gamma > 0.f) || !std::isfinite(gamma)) {
        fail(EF21_EINVAL, "gamma must be finite and > 0");
        return nullptr;
    }
    ef21_ctx *c = new (std::nothrow) ef21_ctx;
    if (!c) {
        fail(EF21_ENOMEM, "host allocation failed");
        return nullptr;
    }
    c->n = n;
    c->d = d;
    c->k = k;
    c->gamma = gamma;
    if (hipGetDevice(&c->device) != hipSuccess) {
        fail(EF21_EHIP, "hipGetDevice failed");
        delete c;
        return nullptr;
    }
    const size_t nd = (size_t)n * d, nk = (size_t)n * k;
    bool ok = hipMalloc((void **)&c->x, sizeof(float) * d) == hipSuccess &&
              hipMalloc((void **)&c->g, sizeof(float) * d) == hipSuccess &&
              hipMalloc((void **)&c->g_i, sizeof(float) * nd) == hipSuccess &&
              hipMalloc((void **)&c->msg_idx, sizeof(int32_t) * nk) == hipSuccess &&
              hipMalloc((void **)&c->msg_val, sizeof(float) * nk) == hipSuccess;
    if (ok) ok = hipMalloc(&c->agg_index, ef21::aggregate_index_bytes(n, d)) == hipSuccess;
    if (ok && use_split(d))
        ok = alloc_split_workspace(&c->topk_ws, ef21::topk_split_workspace_bytes(n, d, k), n, d) == hipSuccess;
    if (ok)
        ok = hipMemset(c->x, 0, sizeof(float) * d) == hipSuccess && hipMemset(c->g, 0, sizeof(float) * d) == hipSuccess &&
             hipMemset(c->g_i, 0, sizeof(float) * nd) == hipSuccess &&
             hipMemset(c->msg_idx, 0, sizeof(int32_t) * nk) == hipSuccess &&
             hipMemset(c->msg_val, 0, sizeof(float) * nk) == hipSuccess && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        free_ctx(c);
        fail(EF21_ENOMEM, "device allocation of the EF21 state failed");
        return nullptr;
    }
    return c;
}

int ef21_destroy(ef21_handle h) {
    if (!h) return EF21_OK;
    hipError_t st = hipStreamSynchronize(h->stream);
    free_ctx(h);
    if (st != hipSuccess) return fail_hip(st, "hipStreamSynchronize");
    return EF21_OK;
}

int ef21_set_stream(ef21_handle h, void *hip_stream) {
    if (int rc = check_handle(h)) return rc;
    h->stream = (hipStream_t)hip_stream;
    return EF21_OK;
}

int ef21_topk(const float *rows, int32_t n, int64_t d, int64_t k, int32_t *out_idx, float *out_val,
              void *hip_stream) {
    if (int rc = check_topk_sizes(n, d, k)) return rc;
    if (!rows || !out_idx || !out_val) return fail(EF21_EINVAL, "rows, out_idx and out_val must not be NULL");
    hipStream_t stream = (hipStream_t)hip_stream;
    void *ws = nullptr;
    if (topk_needs_workspace(d, k)) {
        int dev = 0;
        EF21_HIP(hipGetDevice(&dev));
        const size_t need = ef21::topk_split_workspace_bytes(n, d, k);
        std::lock_guard<std::mutex> lock(g_topk_ws.mu);
        StreamWorkspace *mine = nullptr;
        size_t on_device = 0;
        for (auto &e : g_topk_ws.list) {
            if (e.device != dev) continue;
            ++on_device;
            if (e.stream == stream) mine = &e;
        }
        if (!mine) {
            if (on_device >= kMaxTopkStreams) {             // start over on this device
                EF21_HIP(hipDeviceSynchronize());
                auto &l = g_topk_ws.list;
                for (size_t i = 0; i < l.size();) {
                    if (l[i].device == dev) {
                        (void)hipFree(l[i].ptr);
                        l.erase(l.begin() + (long)i);
                    } else {
                        ++i;
                    }
                }
            }
            StreamWorkspace fresh;
            fresh.device = dev;
            fresh.stream = stream;
            g_topk_ws.list.push_back(fresh);
            mine = &g_topk_ws.list.back();
        }
        if (mine->bytes < need) {
            // earlier calls on this stream may still be using the old block
            EF21_HIP(hipStreamSynchronize(stream));
            (void)hipFree(mine->ptr);
            mine->ptr = nullptr;
            mine->bytes = 0;
            if (hipMalloc(&mine->ptr, need) != hipSuccess) {
                (void)hipGetLastError();
                return fail(EF21_ENOMEM, "hipMalloc of the Top-k workspace failed");
            }
            mine->bytes = need;
            mine->last_n = 0;
        }
        ws = mine->ptr;
        if (mine->last_n != n || mine->last_d != d) {
            hipError_t st = ef21::launch_topk_split_reset(ws, n, d, stream);
            if (st != hipSuccess) return fail_hip(st, "workspace reset launch");
            mine->last_n = n;
            mine->last_d = d;
        }
    }
    ef21::TopkArgs p{rows, nullptr, n, d, k, out_idx, out_val, nullptr};
    return enqueue_topk(p, ws, stream, ef21::Marker());
}

int ef21_topk_static(const float *rows, int32_t n, int64_t d, int64_t k, int32_t *out_idx, float *out_val,
                     void *hip_stream) {
    if (int rc = check_topk_sizes(n, d, k)) return rc;
    if (!rows || !out_idx || !out_val) return fail(EF21_EINVAL, "rows, out_idx and out_val must not be NULL");
    hipStream_t stream = (hipStream_t)hip_stream;
    void *ws = nullptr;
    if (topk_needs_workspace(d, k)) {
        const size_t need = ef21::topk_split_workspace_bytes(n, d, k);
        if (need > kStaticScratchBytes)
            return fail(EF21_EINVAL, "ef21_topk_static: n rows of d entries need " + std::to_string(need) +
                                         " bytes of workspace, the static scratch holds " +
                                         std::to_string(kStaticScratchBytes) + " (use ef21_topk)");
        int dev = 0;
        EF21_HIP(hipGetDevice(&dev));
        if (dev < 0 || dev >= 64) return fail(EF21_ESTATE, "device ordinal out of range");
        {
            std::lock_guard<std::mutex> lock(g_static_ws.mu);
            if (!g_static_ws.ptr[dev]) {
                void *p = nullptr;
                EF21_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
                if (!p) return fail(EF21_EHIP, "hipGetSymbolAddress returned no address for the static scratch");
                g_static_ws.ptr[dev] = p;
            }
            ws = g_static_ws.ptr[dev];
        }
        // The array keeps the last call's contents (of any shape): the control words that must start at zero are
        // cleared by a fill kernel, every call.
        hipError_t st = ef21::launch_topk_split_reset(ws, n, d, stream);
        if (st != hipSuccess) return fail_hip(st, "scratch reset launch");
    }
    ef21::TopkArgs p{rows, nullptr, n, d, k, out_idx, out_val, nullptr};
    return enqueue_topk(p, ws, stream, ef21::Marker());
}

int ef21_set_problem_dense(ef21_handle h, const float *A, const float *y, int64_t m, float lambda) {
    if (int rc = check_handle(h)) return rc;
    if (!A || !y) return fail(EF21_EINVAL, "A and y must not be NULL");
    if (m < 1 || m >= ((int64_t)1 << 31)) return fail(EF21_EINVAL, "m must be in [1, 2^31)");
    if (!(lambda >= 0.f) || !std::isfinite(lambda)) return fail(EF21_EINVAL, "lambda must be finite and >= 0");
    if (int rc = ensure_problem_buffers(h, ef21::logreg_dense_scratch_bytes(h->n, m, h->d))) return rc;
    if (!h->tickets && ef21::small_step_applies(A, h->n, m, h->d, h->k)) {
        const size_t bytes = ef21::small_step_ticket_bytes(h->n);
        if (hipMalloc(&h->tickets, bytes) != hipSuccess) {
            (void)hipGetLastError();
            h->tickets = nullptr;
            return fail(EF21_ENOMEM, "hipMalloc of the iteration's counters failed");
        }
        EF21_HIP(hipMemsetAsync(h->tickets, 0, bytes, h->stream));
    }
    h->kind = kDense;
    h->batch = ef21::RowBatch();
    h->A = A;
    h->y = y;
    h->m = m;
    h->lambda = lambda;
    return EF21_OK;
}

int ef21_set_problem_csr(ef21_handle h, const int64_t *rowptr, const int32_t *col, const float *val,
                         const float *y, int64_t m, float lambda) {
    if (int rc = check_handle(h)) return rc;
    if (!rowptr || !col || !val || !y) return fail(EF21_EINVAL, "rowptr, col, val and y must not be NULL");
    if (m < 1 || m >= ((int64_t)1 << 31)) return fail(EF21_EINVAL, "m must be in [1, 2^31)");
    if (!(lambda >= 0.f) || !std::isfinite(lambda)) return fail(EF21_EINVAL, "lambda must be finite and >= 0");
    if (int rc = ensure_problem_buffers(h, 0)) return rc;
    EF21_HIP(hipStreamSynchronize(h->stream));
    (void)hipFree(h->csr_index);
    h->csr_index = nullptr;
    h->csr_indexed = false;
    int64_t nnz = 0;
    EF21_HIP(hipMemcpy(&nnz, rowptr + (int64_t)h->n * m, sizeof(nnz), hipMemcpyDeviceToHost));
    if (nnz < 0) return fail(EF21_EINVAL, "rowptr[n*m] (the number of entries) is negative");
    const size_t index_bytes = ef21::logreg_csr_index_bytes(h->n, m, h->d, nnz);
    if (index_bytes) {
        if (hipMalloc(&h->csr_index, index_bytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(EF21_ENOMEM, "hipMalloc of the CSR index and column-major copy failed");
        }
        EF21_HIP(ef21::logreg_csr_build_index(rowptr, col, val, h->n, m, h->d, nnz, h->csr_index, h->stream,
                                              &h->csr_indexed));
    }
    h->nnz = nnz;
    h->kind = kCSR;
    h->batch = ef21::RowBatch();
    h->rowptr = rowptr;
    h->col = col;
    h->val = val;
    h->y = y;
    h->m = m;
    h->lambda = lambda;
    return EF21_OK;
}

int ef21_set_loss(ef21_handle h, int loss) {
    if (int rc = check_handle(h)) return rc;
    if (loss != EF21_LOSS_LOGISTIC && loss != EF21_LOSS_LEAST_SQUARES) return fail(EF21_EINVAL, "unknown loss");
    h->loss = loss;
    return EF21_OK;
}

int ef21_set_minibatch(ef21_handle h, const int32_t *rows, int64_t tau) {
    if (int rc = check_handle(h)) return rc;
    if (h->kind == kNone) return fail(EF21_ESTATE, "no problem attached");
    if (tau < 0 || tau > h->m) return fail(EF21_EINVAL, "tau must be in [0, m]");
    if (tau > 0 && !rows) return fail(EF21_EINVAL, "rows is NULL");
    h->batch = ef21::RowBatch();
    if (tau > 0) {
        h->batch.rows = rows;
        h->batch.tau = tau;
    }
    return EF21_OK;
}

int ef21_set_state(ef21_handle h, const float *x, const float *g_i, const float *g) {
    if (int rc = check_handle(h)) return rc;
    const size_t db = sizeof(float) * (size_t)h->d;
    if (x) EF21_HIP(hipMemcpyAsync(h->x, x, db, hipMemcpyDeviceToDevice, h->stream));
    if (g_i) EF21_HIP(hipMemcpyAsync(h->g_i, g_i, db * h->n, hipMemcpyDeviceToDevice, h->stream));
    if (g) {
        EF21_HIP(hipMemcpyAsync(h->g, g, db, hipMemcpyDeviceToDevice, h->stream));
    } else {
        hipError_t st = ef21::launch_mean_rows(h->g_i, h->g, h->n, h->d, h->stream);
        if (st != hipSuccess) return fail_hip(st, "mean kernel launch");
    }
    return EF21_OK;
}

int ef21_get_state(ef21_handle h, float *x, float *g_i, float *g) {
    if (int rc = check_handle(h)) return rc;
    const size_t db = sizeof(float) * (size_t)h->d;
    if (x) EF21_HIP(hipMemcpyAsync(x, h->x, db, hipMemcpyDeviceToDevice, h->stream));
    if (g_i) EF21_HIP(hipMemcpyAsync(g_i, h->g_i, db * h->n, hipMemcpyDeviceToDevice, h->stream));
    if (g) EF21_HIP(hipMemcpyAsync(g, h->g, db, hipMemcpyDeviceToDevice, h->stream));
    return EF21_OK;
}

int ef21_get_messages(ef21_handle h, int32_t *idx, float *val) {
    if (int rc = check_handle(h)) return rc;
    const size_t nk = (size_t)h->n * h->k;
    if (idx) EF21_HIP(hipMemcpyAsync(idx, h->msg_idx, sizeof(int32_t) * nk, hipMemcpyDeviceToDevice, h->stream));
    if (val) EF21_HIP(hipMemcpyAsync(val, h->msg_val, sizeof(float) * nk, hipMemcpyDeviceToDevice, h->stream));
    return EF21_OK;
}

int ef21_local_grad(ef21_handle h, const float *x, float *out_grad) {
    if (int rc = check_handle(h)) return rc;
    if (!out_grad) return fail(EF21_EINVAL, "out_grad must not be NULL");
    if (h->kind == kNone) return fail(EF21_ESTATE, "no problem attached (ef21_set_problem_dense / _csr)");
    record_mark(h, -1);
    return enqueue_local_grad(h, x ? x : h->x, out_grad);
}

// (1/m) A_i^T A_i v_i for every worker (v one row per worker, or one shared row): the gradient kernels with the
// per-row loss z^2 / 2, no regulariser, all rows.
static int enqueue_gram_product(ef21_ctx *c, const float *v, int64_t v_stride, float *out) {
    hipError_t st;
    if (c->kind == kDense)
        st = ef21::launch_logreg_grad_dense(c->A, c->y, v, out, c->n, c->m, c->d, 0.f, c->scratch, c->stream,
                                            ef21::Marker(), nullptr, ef21::kLossHalfSquare, ef21::RowBatch(), v_stride);
    else
        st = ef21::launch_logreg_grad_csr(c->rowptr, c->col, c->val, c->y, v, out, c->n, c->m, c->d, c->nnz, 0.f,
                                          c->csr_indexed ? c->csr_index : nullptr, c->stream, ef21::Marker(),
                                          ef21::kLossHalfSquare, ef21::RowBatch(), v_stride);
    if (st != hipSuccess) return fail_hip(st, "gradient kernel launch");
    return EF21_OK;
}

int ef21_theory_stepsize(ef21_handle h, int32_t iterations, double *gamma, double *L, double *L_i) {
    if (int rc = check_handle(h)) return rc;
    if (h->kind == kNone) return fail(EF21_ESTATE, "no problem attached (ef21_set_problem_dense / _csr)");
    if (iterations < 1 || iterations > 1000000) return fail(EF21_EINVAL, "iterations must be in [1, 10^6]");
    const int32_t n = h->n;
    const int64_t d = h->d;
    // rows 0..n-1: the workers' vectors; row n: the vector of the whole problem; row n+1: its product
    if (!h->power_v) {
        if (hipMalloc((void **)&h->power_v, sizeof(float) * (size_t)(n + 2) * (size_t)d) != hipSuccess ||
            hipMalloc((void **)&h->power_stats, sizeof(double) * 2 * (size_t)(n + 1)) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(h->power_v);
            h->power_v = nullptr;
            h->power_stats = nullptr;
            return fail(EF21_ENOMEM, "hipMalloc of the power iteration's vectors failed");
        }
    }
    float *v = h->power_v;
    double *stats = h->power_stats;
    float *v_all = v + (size_t)n * d, *w_all = v_all + d;
    int rc = EF21_OK;
    hipError_t st = ef21::launch_power_start(v, n + 1, d, h->stream);
    for (int32_t it = 0; it < iterations && st == hipSuccess && rc == EF21_OK; ++it) {
        rc = enqueue_gram_product(h, v, d, h->grad);                         // w_i = (1/m) A_i^T A_i v_i
        if (rc != EF21_OK) break;
        st = ef21::launch_power_step(h->grad, v, n, d, stats, h->stream);
        if (st != hipSuccess) break;
        rc = enqueue_gram_product(h, v_all, 0, h->grad);                     // (1/n) sum_i (1/m) A_i^T A_i v
        if (rc != EF21_OK) break;
        st = ef21::launch_mean_rows(h->grad, w_all, n, d, h->stream);
        if (st != hipSuccess) break;
        st = ef21::launch_power_step(w_all, v_all, 1, d, stats + 2 * (size_t)n, h->stream);
    }
    std::vector<double> host(2 * (size_t)(n + 1));
    if (st == hipSuccess && rc == EF21_OK)
        st = hipMemcpyAsync(host.data(), stats, sizeof(double) * host.size(), hipMemcpyDeviceToHost, h->stream);
    const hipError_t sync = hipStreamSynchronize(h->stream);
    if (rc != EF21_OK) return rc;
    if (st != hipSuccess) return fail_hip(st, "power iteration");
    if (sync != hipSuccess) return fail_hip(sync, "power iteration");
    // curvature of the per-row loss in its margin, and of lambda t^2 / (1 + t^2)
    const double c = h->loss == EF21_LOSS_LEAST_SQUARES ? 2.0 : 0.25, reg = 2.0 * (double)h->lambda;
    double sum_sq = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        const double Li = c * host[2 * (size_t)i + 1] + reg;
        if (L_i) L_i[i] = Li;
        sum_sq += Li * Li;
    }
    const double L_all = c * host[2 * (size_t)n + 1] + reg;
    if (L) *L = L_all;
    if (gamma) {
        const double alpha = (double)h->k / (double)d, r = sqrt(1.0 - alpha);
        *gamma = 1.0 / (L_all + sqrt(sum_sq / n) * ((1.0 + r) / alpha - 1.0));
    }
    return EF21_OK;
}

// Buffers of Algorithm 3, allocated by the first EF21_PLUS step of a handle.
static int ensure_plus_buffers(ef21_ctx *c) {
    if (c->plus_bm) return EF21_OK;
    const size_t nk = (size_t)c->n * (size_t)c->k;
    EF21_HIP(hipStreamSynchronize(c->stream));
    if (hipMalloc((void **)&c->plus_idx, sizeof(int32_t) * 2 * nk) != hipSuccess ||
        hipMalloc((void **)&c->plus_val, sizeof(float) * 2 * nk) != hipSuccess ||
        hipMalloc(&c->plus_scratch, ef21::plus_scratch_bytes(c->n, c->d, c->k)) != hipSuccess ||
        hipMalloc((void **)&c->plus_branch, sizeof(int32_t) * (size_t)c->n) != hipSuccess ||
        hipMalloc((void **)&c->plus_bm, sizeof(double) * 2 * (size_t)c->n) != hipSuccess ||
        (c->topk_ws && c->k > 1 &&
         alloc_split_workspace(&c->topk_ws2, ef21::topk_split_workspace_bytes(c->n, c->d, c->k), c->n, c->d) != hipSuccess)) {
        (void)hipGetLastError();
        (void)hipFree(c->plus_idx);
        (void)hipFree(c->plus_val);
        (void)hipFree(c->plus_scratch);
        (void)hipFree(c->plus_branch);
        (void)hipFree(c->plus_bm);
        (void)hipFree(c->topk_ws2);
        c->topk_ws2 = nullptr;
        c->plus_idx = nullptr;
        c->plus_val = nullptr;
        c->plus_scratch = nullptr;
        c->plus_branch = nullptr;
        c->plus_bm = nullptr;
        return fail(EF21_ENOMEM, "hipMalloc of the EF21+ buffers failed");
    }
    return EF21_OK;
}

// Lines 5 to 8 and 10 of Algorithm 3 for all workers (the model step is the caller's).
static int enqueue_plus(ef21_ctx *h, const float *grads, const ef21::Marker &mk) {
    const size_t nk = (size_t)h->n * (size_t)h->k;
    int32_t *idx_b = h->plus_idx, *idx_m = h->plus_idx + nk;
    float *val_b = h->plus_val, *val_m = h->plus_val + nk;
    ef21::TopkArgs plain{grads, nullptr, h->n, h->d, h->k, idx_b, val_b, nullptr};        // line 5: C(s)
    plain.warm = 2;
    ef21::TopkArgs markov{grads, h->g_i, h->n, h->d, h->k, idx_m, val_m, nullptr};        // line 6: C(s - g_i)
    markov.warm = 1;
    int64_t norm_chunks = 0;
    hipError_t st;
    if (h->topk_ws2) {
        // long rows: both selections and the two squared norms of line 7 from ONE pass over s and g_i
        plain.warm = 1;           // each workspace keeps its own thresholds
        st = ef21::launch_topk_split_pair(plain, markov, h->topk_ws2, h->topk_ws, h->plus_scratch, h->stream, mk);
        if (st != hipSuccess) return fail_hip(st, "Top-k kernel launch");
        norm_chunks = ef21::topk_split_slots(h->n, h->d);
    } else {
        if (int rc = enqueue_topk(plain, h->topk_ws, h->stream, mk)) return rc;
        if (int rc = enqueue_topk(markov, h->topk_ws, h->stream, mk)) return rc;
    }
    st = ef21::launch_plus_choose(grads, h->g_i, h->n, h->d, h->k, idx_b, val_b, idx_m, val_m, h->plus_scratch,
                                  h->plus_branch, h->plus_bm, h->msg_idx, h->msg_val, h->stream,
                                  norm_chunks);                                            // lines 7 and 8
    if (st == hipSuccess) st = ef21::launch_mean_rows(h->g_i, h->g, h->n, h->d, h->stream);   // line 10
    mk(ef21::K_PLUS);
    if (st != hipSuccess) return fail_hip(st, "EF21+ kernel launch");
    return EF21_OK;
}

// One round of Algorithm 4 (EF) on the handle: the errors e_i live in g_i, g receives (1/n) sum_i w_i.
static int enqueue_classic_ef(ef21_ctx *h, const float *grads, const ef21::Marker &mk) {
    hipError_t st = ef21::launch_ef_accumulate(grads, h->g_i, h->n, h->d, h->gamma, h->stream);   // p_i over e_i
    mk(ef21::K_PLUS);
    if (st != hipSuccess) return fail_hip(st, "EF accumulation launch");
    ef21::TopkArgs p{h->g_i, nullptr, h->n, h->d, h->k, h->msg_idx, h->msg_val, nullptr};            // w_i = C(p_i)
    p.warm = 1;
    bool index_ready = false;
    want_message_index(h, &p);
    if (int rc = enqueue_topk(p, h->topk_ws, h->stream, mk, &index_ready)) return rc;
    st = ef21::launch_ef_clear_kept(h->msg_idx, h->n, h->k, h->g_i, h->d, h->stream);               // e_i = p_i - w_i
    if (st == hipSuccess) st = ef21::launch_fill_zero(h->g, h->d, h->stream);
    mk(ef21::K_PLUS);
    if (st != hipSuccess) return fail_hip(st, "EF error update launch");
    st = ef21::launch_aggregate(h->msg_idx, h->msg_val, h->n, h->k, h->d, h->g, h->x, 1.0f, h->agg_index,
                                h->stream, index_ready);                                            // x - mean w
    mk(ef21::K_MODEL_STEP);
    if (st != hipSuccess) return fail_hip(st, "aggregation launch");
    return EF21_OK;
}

int ef21_step(ef21_handle h, const float *grads, uint32_t flags) {
    if (int rc = check_handle(h)) return rc;
    if (flags & ~(uint32_t)(EF21_ORDER_STEP_FIRST | EF21_PLUS | EF21_CLASSIC_EF | EF21_ONE_LAUNCH))
        return fail(EF21_EINVAL, "unknown flags");
    if ((flags & EF21_CLASSIC_EF) && (flags & (EF21_ORDER_STEP_FIRST | EF21_PLUS)))
        return fail(EF21_EINVAL, "EF21_CLASSIC_EF combines with neither an order nor EF21_PLUS");
    if (!grads && h->kind == kNone)
        return fail(EF21_ESTATE, "grads is NULL and no problem is attached to compute them from");
    if (flags & EF21_CLASSIC_EF) {
        const ef21::Marker mk0 = marker_of(h);
        mk0(-1);
        if (!grads) {
            if (int rc = enqueue_local_grad(h, h->x, h->grad)) return rc;
            grads = h->grad;
        }
        return enqueue_classic_ef(h, grads, mk0);
    }
    const bool step_first = (flags & EF21_ORDER_STEP_FIRST) != 0;
    const bool plus = (flags & EF21_PLUS) != 0;
    if (plus)
        if (int rc = ensure_plus_buffers(h)) return rc;
    const ef21::Marker mk = marker_of(h);
    mk(-1);
    if (step_first) {   // Algorithm 2, line 3
        hipError_t st = ef21::launch_model_step(h->x, h->g, h->d, h->gamma, h->stream);
        mk(ef21::K_MODEL_STEP);
        if (st != hipSuccess) return fail_hip(st, "model step launch");
    }
    if (plus) {
        if (!grads) {
            if (int rc = enqueue_local_grad(h, h->x, h->grad)) return rc;
            grads = h->grad;
        }
        if (int rc = enqueue_plus(h, grads, mk)) return rc;
        if (!step_first) {
            hipError_t st = ef21::launch_model_step(h->x, h->g, h->d, h->gamma, h->stream);
            mk(ef21::K_MODEL_STEP);
            if (st != hipSuccess) return fail_hip(st, "model step launch");
        }
        return EF21_OK;
    }
    if (!grads && h->kind == kDense && h->tickets && h->batch.tau == 0 && (flags & EF21_ONE_LAUNCH) &&
        ef21::small_step_applies(h->A, h->n, h->m, h->d, h->k)) {
        // lines 5, 6, 8 (and 3) in one launch
        hipError_t st = ef21::launch_small_step(h->A, h->y, h->x, h->g, h->g_i, h->n, h->m, h->d, h->k, h->lambda,
                                                h->gamma, h->loss, !step_first, h->scratch, h->tickets, h->msg_idx,
                                                h->msg_val, h->stream);
        mk(ef21::K_SMALL_STEP);
        if (st != hipSuccess) return fail_hip(st, "iteration kernel launch");
        return EF21_OK;
    }
    ef21::GradParts parts;
    if (!grads) {
        const bool row_kernel = !(use_split(h->d) && h->topk_ws);
        if (int rc = enqueue_local_grad(h, h->x, h->grad, row_kernel ? &parts : nullptr)) return rc;
        grads = h->grad;
    }
    // lines 5 and 6: Top-k of grads - g_i, fused with the update of g_i
    ef21::TopkArgs p{grads, h->g_i, h->n, h->d, h->k, h->msg_idx, h->msg_val, h->g_i, parts};
    p.warm = 1;
    bool index_ready = false;
    want_message_index(h, &p);
    if (int rc = enqueue_topk(p, h->topk_ws, h->stream, mk, &index_ready)) return rc;
    // line 8 from the messages, and (default order) line 3 in the same pass over the coordinates
    hipError_t st = ef21::launch_aggregate(h->msg_idx, h->msg_val, h->n, h->k, h->d, h->g, step_first ? nullptr : h->x,
                                           h->gamma, h->agg_index, h->stream, index_ready);
    mk(ef21::K_MODEL_STEP);
    if (st != hipSuccess) return fail_hip(st, "aggregation launch");
    return EF21_OK;
}

int ef21_get_choices(ef21_handle h, int32_t *branch, double *distortions) {
    if (int rc = check_handle(h)) return rc;
    if (!h->plus_bm) return fail(EF21_ESTATE, "no EF21_PLUS step has been taken on this handle");
    if (branch)
        EF21_HIP(hipMemcpyAsync(branch, h->plus_branch, sizeof(int32_t) * (size_t)h->n, hipMemcpyDeviceToDevice,
                                h->stream));
    if (distortions)
        EF21_HIP(hipMemcpyAsync(distortions, h->plus_bm, sizeof(double) * 2 * (size_t)h->n, hipMemcpyDeviceToDevice,
                                h->stream));
    return EF21_OK;
}

int ef21_set_timing(ef21_handle h, int enabled) {
    if (int rc = check_handle(h)) return rc;
    EF21_HIP(hipStreamSynchronize(h->stream));
    drain_timing(h);
    h->timing.on = enabled != 0;
    return EF21_OK;
}

int ef21_get_timing(ef21_handle h, double *ms, int64_t *launches, int reset) {
    if (int rc = check_handle(h)) return rc;
    EF21_HIP(hipStreamSynchronize(h->stream));
    drain_timing(h);
    for (int i = 0; i < EF21_K_COUNT; ++i) {
        if (ms) ms[i] = h->timing.ms[i];
        if (launches) launches[i] = h->timing.launches[i];
        if (reset) {
            h->timing.ms[i] = 0.0;
            h->timing.launches[i] = 0;
        }
    }
    return EF21_OK;
}

static int check_hbm_args(const void *a, const void *b, int64_t bytes) {
    if (!a || !b) return fail(EF21_EINVAL, "pointers must not be NULL");
    if (bytes < 16 || bytes % 16 != 0) return fail(EF21_EINVAL, "bytes must be a positive multiple of 16");
    if ((uintptr_t)a % 16 != 0 || (uintptr_t)b % 4 != 0) return fail(EF21_EINVAL, "buffers must be 16-byte aligned");
    return EF21_OK;
}

int ef21_hbm_read(const void *src, int64_t bytes, float *sink, void *hip_stream) {
    if (int rc = check_hbm_args(src, sink, bytes)) return rc;
    EF21_HIP(ef21::launch_hbm_read(src, bytes / 16, sink, (hipStream_t)hip_stream));
    return EF21_OK;
}

int ef21_hbm_copy(void *dst, const void *src, int64_t bytes, void *hip_stream) {
    if (int rc = check_hbm_args(src, dst, bytes)) return rc;
    if ((uintptr_t)dst % 16 != 0) return fail(EF21_EINVAL, "buffers must be 16-byte aligned");
    EF21_HIP(ef21::launch_hbm_copy(dst, src, bytes / 16, (hipStream_t)hip_stream));
    return EF21_OK;
}

const char *ef21_kernel_name(int kernel_class) {
    static const char *names[EF21_K_COUNT] = {"grad_main",   "grad_aux",   "topk_row",  "topk_collect", "topk_select",
                                              "topk_refine", "topk_count", "topk_emit", "model_step",
                                              "plus",        "small_step"};
    return (kernel_class >= 0 && kernel_class < EF21_K_COUNT) ? names[kernel_class] : "";
}

}  // extern "C"
