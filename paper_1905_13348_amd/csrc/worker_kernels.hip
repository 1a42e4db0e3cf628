// Worker selection (Section 4.1, Case I: the policy returns the variant and the worker that serves
// the query; Section 6.4 counts the choice of the worker as the second decision on the critical
// path).  An Active variant is served by the least-loaded worker that runs an instance of it, an
// Inactive one by the least-utilised worker that has its target hardware.
//
// The worker depends on the variant and its tier only, not on the query.  So these kernels keep a
// worker per variant up to date (k_worker_tables, from the reports applied by k_worker_report) and
// copy it next to every step of the staircase indexes (k_step_workers); the lookup kernel then
// fetches the worker of an answer with the same gather that fetches its row.
#include "internal.h"

namespace infaas {

namespace {

constexpr int kThreads = 256;

// util[worker_idx[i]] = util_new[i] (i < n) and load of instance inst_idx[j] = load_new[j] (j < m);
// entries outside the tables or with a negative value are skipped; the indices must be distinct.
__global__ __launch_bounds__(kThreads) void k_worker_report(WorkerView wv, int32_t n, const int32_t *__restrict__ worker_idx,
                                                            const int32_t *__restrict__ util_new, int32_t m,
                                                            const int32_t *__restrict__ inst_idx,
                                                            const int32_t *__restrict__ load_new)
{
    const int32_t i = (int32_t)(blockIdx.x * kThreads + threadIdx.x);
    if (i < n) {
        const int32_t w = worker_idx[i], u = util_new[i];
        if ((uint32_t)w < (uint32_t)wv.W && u >= 0) wv.util[w] = u;
    } else if (i - n < m) {
        const int32_t j = inst_idx[i - n], l = load_new[i - n];
        if ((uint32_t)j < (uint32_t)wv.I && l >= 0) wv.inst_load[wv.inst_pos[j]] = l;
    }
}

// State of instance inst_idx[i] = state[i]; a loaded instance is Active (1), Overloaded (2) or Interfered (3).
__global__ __launch_bounds__(kThreads) void k_instance_state_report(WorkerView wv, int32_t n, const int32_t *__restrict__ inst_idx,
                                                                   const int32_t *__restrict__ state)
{
    const int32_t i = (int32_t)(blockIdx.x * kThreads + threadIdx.x);
    if (i >= n) return;
    const int32_t j = inst_idx[i], c = state[i];
    if ((uint32_t)j < (uint32_t)wv.I && c >= 1 && c <= 3) wv.inst_state[wv.inst_pos[j]] = c;
}

// One lane per variant: its state as its instances give it (Section 4 keeps the state machine per
// variant instance): Inactive when it runs nowhere, Active when some instance is, else Overloaded when
// some instance is, else Interfered.
__global__ __launch_bounds__(kThreads) void k_derive_states(WorkerView wv)
{
    const int32_t v = (int32_t)(blockIdx.x * kThreads + threadIdx.x);
    if (v >= wv.V) return;
    const int32_t lo = wv.inst_off[v], hi = wv.inst_off[v + 1];
    bool active = false, overloaded = false;
    for (int32_t i = lo; i < hi; ++i) {
        const int32_t c = wv.inst_state[i];
        active = active || c == 1;
        overloaded = overloaded || c == 2;
    }
    wv.derived[v] = hi == lo ? 0 : (active ? 1 : (overloaded ? 2 : 3));
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off; off >>= 1) {
        const uint64_t o = __shfl_xor(v, off);
        v = o < v ? o : v;
    }
    return v;
}

// One workgroup per hardware class: the worker with the smallest (utilisation, number).
__global__ __launch_bounds__(kThreads) void k_best_per_class(WorkerView wv)
{
    __shared__ uint64_t s_best[kThreads / 64];
    const int32_t c = (int32_t)blockIdx.x;
    const int32_t lo = wv.cls_off[c], hi = wv.cls_off[c + 1];
    uint64_t best = ~0ull;
    for (int32_t i = lo + (int32_t)threadIdx.x; i < hi; i += kThreads) {
        const int32_t w = wv.cls_worker[i];
        const uint64_t key = ((uint64_t)(uint32_t)wv.util[w] << 32) | (uint32_t)w;   // utilisation is never negative
        best = key < best ? key : best;
    }
    best = wave_min_u64(best);
    if ((threadIdx.x & 63) == 0) s_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 1; k < kThreads / 64; ++k) best = s_best[k] < best ? s_best[k] : best;
        wv.best_cls[c] = hi > lo ? (int32_t)(uint32_t)best : -1;
    }
}

// One lane per variant: the worker of its instance with the smallest (load, worker) -- of its Active
// instances, when the instances carry states -- and the best worker of its hardware class.
__global__ __launch_bounds__(kThreads) void k_worker_tables(WorkerView wv)
{
    const int32_t v = (int32_t)(blockIdx.x * kThreads + threadIdx.x);
    if (v >= wv.V) return;
    uint64_t best = ~0ull;
    for (int32_t i = wv.inst_off[v]; i < wv.inst_off[v + 1]; ++i) {
        if (wv.inst_state && wv.inst_state[i] != 1) continue;
        const uint64_t key = ((uint64_t)(uint32_t)wv.inst_load[i] << 32) | (uint32_t)wv.inst_worker[i];
        best = key < best ? key : best;
    }
    wv.row_worker[v] = best != ~0ull ? (int32_t)(uint32_t)best : -1;
    const int32_t c = wv.var_cls[v];
    wv.row_worker[wv.V + v] = c >= 0 ? wv.best_cls[c] : -1;
}

// Entries of step_row that a slice reserved but could not fill hold no row: anything outside
// 0..num_rows-1 gets no worker.
__global__ __launch_bounds__(kThreads) void k_step_workers(IndexView ix, const int32_t *__restrict__ row_worker,
                                                           int32_t num_rows)
{
    const uint32_t j = blockIdx.x * kThreads + threadIdx.x;
    const uint32_t steps = ix.ctrl[kCtlSteps];   // entries of step_row in use (entry 0 included)
    if (j >= steps || j >= ix.step_cap) return;
    const int32_t row = ix.step_row[j];
    ix.step_worker[j] = (uint32_t)row < (uint32_t)num_rows ? row_worker[row] : -1;
}

// One lane per (slice, hot step): the 16-bit copy of the step's worker that the lookup kernel keeps
// in LDS.  Places past the slice's last step are never read by the lookup.
__global__ __launch_bounds__(kThreads) void k_hot_workers(IndexView ix, int32_t num_slices)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= (uint32_t)num_slices * ix.hot_rows) return;
    const uint32_t s = i / ix.hot_rows, step = i - s * ix.hot_rows;
    const uint4 hdr = ix.hdr[s];
    const uint32_t at = hdr.z + step;   // the slice's first entry in step_row / step_worker, plus the step
    const int32_t w = ((hdr.y & kHdrPark) || at >= ix.step_cap) ? -1 : ix.step_worker[at];
    ix.hot_worker[i] = (uint32_t)w < 0xFFFFu ? (uint16_t)w : (uint16_t)0xFFFFu;
}

}  // namespace

hipError_t launch_hot_workers(const IndexView &ix, int32_t num_slices, hipStream_t st, const LaunchEvents *ev)
{
    const int64_t n = (int64_t)num_slices * ix.hot_rows;
    if (!ix.hot_worker || n <= 0) return hipSuccess;
    return launch_kernel(ev, k_hot_workers, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, ix,
                         num_slices);
}

hipError_t launch_worker_report(const WorkerView &wv, int32_t n, const int32_t *worker_idx, const int32_t *util,
                                int32_t m, const int32_t *inst_idx, const int32_t *load, hipStream_t st,
                                const LaunchEvents *ev)
{
    const int64_t total = (int64_t)n + m;
    if (total <= 0) return hipSuccess;
    return launch_kernel(ev, k_worker_report, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                         wv, n, worker_idx, util, m, inst_idx, load);
}

hipError_t launch_instance_state_report(const WorkerView &wv, int32_t n, const int32_t *inst_idx, const int32_t *state,
                                        hipStream_t st, const LaunchEvents *ev)
{
    if (n <= 0 || !wv.inst_state) return hipSuccess;
    return launch_kernel(ev, k_instance_state_report, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                         wv, n, inst_idx, state);
}

hipError_t launch_derive_states(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev)
{
    if (wv.V <= 0 || !wv.inst_state || !wv.derived) return hipSuccess;
    return launch_kernel(ev, k_derive_states, dim3((unsigned)((wv.V + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, wv);
}

hipError_t launch_best_per_class(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev)
{
    if (wv.H <= 0) return hipSuccess;
    return launch_kernel(ev, k_best_per_class, dim3((unsigned)wv.H), dim3(kThreads), 0, st, wv);
}

hipError_t launch_worker_tables(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev)
{
    if (wv.V <= 0) return hipSuccess;
    return launch_kernel(ev, k_worker_tables, dim3((unsigned)((wv.V + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, wv);
}

hipError_t launch_step_workers(const IndexView &ix, const int32_t *row_worker, int32_t num_rows, hipStream_t st,
                               const LaunchEvents *ev)
{
    // the number of steps in use is known on the device only: one lane per entry there is room for
    return launch_kernel(ev, k_step_workers, dim3((ix.step_cap + kThreads - 1) / kThreads), dim3(kThreads), 0, st, ix,
                         row_worker, num_rows);
}

}  // namespace infaas
