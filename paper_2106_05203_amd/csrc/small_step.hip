// One launch per iteration of Algorithm 2 for problems whose iteration is bound by launch latency rather than
// by bandwidth (dense rows, d <= 1024, a few MB of data): lines 5, 6, 8 and 3 in one kernel.
//
//   every workgroup     four row blocks of one worker's gradient (the code of the gradient kernel, so the
//                       partial sums are the same bits), then a ticket on the worker's counter;
//   the worker's last   finishes the sums to grad f_i, forms grad f_i - g_i, selects Top-k, writes the message
//   workgroup           and updates g_i (the code of the row Top-k kernel), then a ticket on the common counter;
//   the last of those   adds the messages to g in worker order and takes the model step.
//
// Nobody waits: a workgroup that is not the last to draw its ticket simply ends, so the kernel cannot hang.
// The tickets are device-scope atomics between device-scope fences (release before the ticket, acquire after
// it), which is what makes one workgroup's stores visible to another on a different compute die.
#include "device_utils.h"
#include "kernels.h"
#include "logreg_dense_block.h"
#include "topk_row_impl.h"

namespace ef21 {
namespace {

constexpr int kBlocksPerWg = kRowThreads / kDenseThreads;   // 4 row blocks per workgroup of 1024 threads
constexpr int kMaxCols = 1024;                              // d of the fused iteration
constexpr int kMaxEntries = 2048;                           // n * k
constexpr int kMaxAddSteps = 512;                           // n * ceil(k / 64), the adding wavefront's steps
constexpr int64_t kMaxProblem = (int64_t)1 << 24;           // n * m * d

struct SmallArgs {
    const float *A, *y;
    float *x, *g, *g_i, *part;
    int32_t *msg_idx;
    float *msg_val;
    uint32_t *tickets;        // [n + 1], zero between launches
    int32_t n;
    int64_t m, d, k, rows_per_wg, chunks;
    float lambda, inv_n, neg_gamma;
    int loss, step;           // step != 0: line 3 after line 8
};

// All threads of the workgroup call.  Publishes what the workgroup has stored, draws a ticket of `counter`, and
// returns true in the workgroup that drew the last of `tickets` (it may then read what the others published).
// One thread fences for the workgroup: the barriers order the other threads' accesses against its fences (the
// release and acquire are cumulative), and the device-scope fences write back and invalidate caches that the
// whole workgroup shares, so one of each is enough and sixteen wavefronts' worth would only queue up.
__device__ __forceinline__ bool draw_ticket(uint32_t *counter, uint32_t tickets, uint32_t *flag) {
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();                                     // release
        const uint32_t drawn = atomicAdd(counter, 1u);
        __threadfence();                                     // acquire
        *flag = drawn == tickets - 1u ? 1u : 0u;
    }
    __syncthreads();
    return *flag != 0u;
}

template <int VEC, int NQ>
__global__ __launch_bounds__(kRowThreads) void small_step_kernel(SmallArgs a) {
    __shared__ RowShared s;
    __shared__ float red[kBlocksPerWg][NQ * kWave * VEC];
    __shared__ float cache[kMaxCols];
    __shared__ int32_t m_idx[kMaxEntries];
    __shared__ float m_val[kMaxEntries];
    __shared__ uint32_t last;
    const int tid = threadIdx.x;
    const int64_t worker = blockIdx.y;

    // ---- line 5, first half: row blocks of grad f_i
    {
        const int vb = tid / kDenseThreads;
        const int64_t chunk = (int64_t)blockIdx.x * kBlocksPerWg + vb;
        dense_block<VEC, NQ, dense_rows_in_flight<VEC, NQ>(), false>(
            a.A, a.y, a.x, a.part, a.m, a.d, a.rows_per_wg, a.loss, nullptr, a.m, worker, chunk, a.chunks,
            (tid / kWave) % kDenseWaves, tid % kDenseThreads, chunk < a.chunks, red[vb]);
    }
    if (!draw_ticket(&a.tickets[worker], gridDim.x, &last)) return;     // the partial sums of the others, or done

    // ---- lines 5 and 6 for this worker
    {
        TopkArgs p{nullptr, a.g_i, a.n, a.d, a.k, a.msg_idx, a.msg_val, a.g_i,
                   GradParts{a.part, a.chunks, a.m, a.x, a.lambda}};
        row_topk_parts<true>(s, cache, p, worker);
    }
    if (!draw_ticket(&a.tickets[a.n], (uint32_t)a.n, &last)) return;      // all messages, or done

    // ---- line 8, then line 3: the messages staged in LDS, ONE wavefront adds them worker by worker (positions
    // inside a message are distinct, a wavefront's LDS accesses execute in program order)
    const int64_t total = (int64_t)a.n * a.k;
    for (int64_t t = tid; t < total; t += kRowThreads) {
        m_idx[t] = a.msg_idx[t];
        m_val[t] = a.msg_val[t];
    }
    for (int64_t j = tid; j < a.d; j += kRowThreads) cache[j] = 0.f;
    if (tid <= a.n) a.tickets[tid] = 0u;                    // n + 1 <= 1024: every ticket has been drawn
    const float gj = tid < a.d ? a.g[tid] : 0.f;            // d <= 1024: one coordinate per thread
    const float xj = a.step && tid < a.d ? a.x[tid] : 0.f;
    __syncthreads();
    if (tid < kWave) {
        for (int32_t w = 0; w < a.n; ++w) {
            for (int64_t i0 = 0; i0 < a.k; i0 += kWave) {
                const int64_t i = i0 + tid;
                if (i < a.k) cache[m_idx[w * a.k + i]] += m_val[w * a.k + i];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
    __syncthreads();
    if (tid < a.d) {
        const float gn = fmaf(cache[tid], a.inv_n, gj);
        a.g[tid] = gn;
        if (a.step) a.x[tid] = fmaf(a.neg_gamma, gn, xj);
    }
}

template <int VEC, int NQ>
void launch(const SmallArgs &a, hipStream_t stream) {
    const dim3 grid((unsigned)((a.chunks + kBlocksPerWg - 1) / kBlocksPerWg), (unsigned)a.n);
    hipLaunchKernelGGL((small_step_kernel<VEC, NQ>), grid, dim3(kRowThreads), 0, stream, a);
}

}  // namespace

bool small_step_applies(const float *A, int32_t n, int64_t m, int64_t d, int64_t k) {
    const bool vec4 = (d % 4 == 0) && ((uintptr_t)A % 16 == 0);
    const DenseVariant dv = dense_variant(d, vec4);
    return d <= kMaxCols && dv.vec != 0 && dv.vec * dv.nq <= 16 && n < kRowThreads && (int64_t)n * k <= kMaxEntries &&
           (int64_t)n * ((k + kWave - 1) / kWave) <= kMaxAddSteps && (int64_t)n * m * d <= kMaxProblem;
}

size_t small_step_ticket_bytes(int32_t n) { return sizeof(uint32_t) * ((size_t)n + 1); }

hipError_t launch_small_step(const float *A, const float *y, float *x, float *g, float *g_i, int32_t n, int64_t m,
                             int64_t d, int64_t k, float lambda, float gamma, int loss, bool take_step, void *scratch,
                             void *tickets, int32_t *msg_idx, float *msg_val, hipStream_t stream) {
    if (!small_step_applies(A, n, m, d, k)) return hipErrorInvalidValue;
    const DensePlan pl = dense_plan(n, m);
    const SmallArgs a{A, y, x, g, g_i, (float *)scratch, msg_idx, msg_val, (uint32_t *)tickets, n, m, d, k,
                      pl.rows_per_wg, pl.chunks, lambda, 1.0f / (float)n, -gamma, loss, take_step ? 1 : 0};
    const bool vec4 = (d % 4 == 0) && ((uintptr_t)A % 16 == 0);
    const DenseVariant dv = dense_variant(d, vec4);
    switch (dv.vec * 100 + dv.nq) {
        case 401: launch<4, 1>(a, stream); break;
        case 402: launch<4, 2>(a, stream); break;
        case 404: launch<4, 4>(a, stream); break;
        case 102: launch<1, 2>(a, stream); break;
        case 108: launch<1, 8>(a, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace ef21
