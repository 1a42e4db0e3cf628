/*
 * infaas_sel -- batched per-query model-variant selection on one AMD Instinct MI355X.
 *
 * The operation is the variant choice that INFaaS (arxiv 1905.13348) makes on the
 * critical path of every query (Section 4.1, "Case I: on arrival of a query"): given
 * the query's requirements, pick the registered variant of the query's application
 * that meets them at the lowest cost (the cheapest-choice objective of Section 2.2,
 * Tables 2 and 3), taking the variants' current load into account (Section 4), or
 * report that no variant can meet them.  Here millions of such decisions are made per
 * call, on the GPU, with integer arithmetic only.
 *
 * Per query q = (task, slo_us, min_acc_bp, batch_idx) the result is the row v of the
 * variant table that minimises the lexicographic key (cost[v][b], lat_us[v][b], v)
 * among the rows with
 *       task_id[v] == task,
 *       acc_bp[v]  >= min_acc_bp,
 *       lat_us[v][b] + queue_us[v] <= slo_us        (exact sum, never wraps),
 * where b = batch_idx, or -1 when no row qualifies (also for a task or batch index
 * outside the table and for a negative slo_us).
 *
 * Further down: the suggestion of the closest variant when nothing qualifies
 * (infaas_sel_select_closest), the state-aware form of the same decision
 * (infaas_sel_load_states / _update_state / _select_tiered), the worker that serves the
 * chosen variant (infaas_sel_load_workers / _update_workers / _select_workers) and the
 * decisions on a change in load, Case II of Section 4.2 (infaas_sel_load_scaling /
 * infaas_sel_scale / infaas_sel_scale_down).  They follow the conventions stated here.
 *
 * Plain C ABI: opaque handle, plain pointers and sizes.  Each pointer below is marked
 * HOST or DEVICE.  Nothing here allocates or frees memory the caller passed in.
 *
 * Threading / ordering: a handle is not thread-safe.  The calls that take a hip_stream
 * (reports, selections, scaling decisions) only ENQUEUE work on that stream and return;
 * the outputs are valid once the caller has synchronised it.  Work enqueued on
 * one handle must be ordered by the caller (same stream, or events between streams),
 * because all calls share the handle's table and scratch memory.
 */
#ifndef INFAAS_SEL_H
#define INFAAS_SEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct infaas_sel infaas_sel_t; /* opaque; owned by the library */

/* Status codes: 0 on success, negative on failure.  No call aborts or throws. */
enum {
    INFAAS_SEL_OK = 0,
    INFAAS_SEL_ERR_INVALID_ARG = -1,  /* null pointer, negative size, bad config */
    INFAAS_SEL_ERR_NOT_LOADED = -2,   /* select / update_load before load_variants */
    INFAAS_SEL_ERR_OUT_OF_RANGE = -3, /* a table value outside its documented range */
    INFAAS_SEL_ERR_HIP = -4,          /* a HIP runtime call failed */
    INFAAS_SEL_ERR_OOM = -5           /* host or device allocation failed */
};

/* infaas_sel_config.flags, bits 0-3: which search runs inside infaas_sel_select. */
enum {
    /* Default: the staircase index (per slice, the variants no cheaper variant dominates; a
     * query is two binary searches and a bit-set intersection), mirrored in one compute unit's
     * LDS when it fits; when it does not, large batches are binned by groups of tasks whose part of
     * the index fits and looked up group by group, small ones read it from global memory.  Queries the index cannot decide
     * (its per-slice capacity was exceeded) are finished by a rank-ordered scan inside the same
     * kernel, so results never depend on the engine.  If more than half of the slices exceed the
     * capacity when the table is loaded, the exhaustive scan is used instead. */
    INFAAS_SEL_ENGINE_AUTO = 0,
    /* Exhaustive scan only: queries bucketed by (task, batch) slice, slice staged in LDS,
     * feasibility filter and wavefront min-reduction over every variant of the slice. */
    INFAAS_SEL_ENGINE_SCAN = 1,
    /* Staircase index always. */
    INFAAS_SEL_ENGINE_INDEX = 2
};
#define INFAAS_SEL_ENGINE_MASK 0xFu

typedef struct {
    int32_t num_tasks;          /* T >= 1; task ids are 0..T-1 */
    int32_t num_batch_sizes;    /* B, 1..64; queries carry an index 0..B-1 */
    const int32_t *batch_sizes; /* HOST [B], copied, informational (may be NULL) */
    int32_t device;             /* HIP device ordinal the handle lives on */
    uint32_t flags;             /* INFAAS_SEL_ENGINE_* */
    int32_t lds_segment_limit;  /* variants of one (task, batch) slice the scan stages in LDS
                                   at once; larger slices are split across workgroups and the
                                   partial minima merged device-wide.  0 = default (4096);
                                   allowed 64..8192, rounded down to a multiple of 64. */
} infaas_sel_config;

/*
 * Create a handle on cfg->device.  *out is set only on success.
 * Errors: INVALID_ARG (null, T < 1, B outside 1..64, T*B > 2^24, bad flags/limit),
 *         HIP, OOM.
 */
int infaas_sel_create(const infaas_sel_config *cfg, infaas_sel_t **out);

/*
 * Register the variant table (the static profiles and the initial load that the paper
 * keeps in its Metadata Store, Sections 3.2 and 5).  All arrays are HOST memory and are
 * copied; rows may come in any order and row numbers are the variant indices that
 * infaas_sel_select returns and infaas_sel_update_load takes.
 *   task_id  [V]    0..T-1
 *   acc_bp   [V]    accuracy in basis points, any int32
 *   lat_us   [V*B]  row-major [v][b], profiled latency at batch_sizes[b], >= 0
 *   cost     [V*B]  row-major [v][b], cost of one query at that batch size, >= 0
 *   queue_us [V]    current queueing delay, >= 0
 * Synchronous: returns after the table is resident on the device.  Replaces any table
 * loaded before.  V = 0 is allowed (every query then answers -1).
 * Errors: INVALID_ARG, OUT_OF_RANGE (task id outside 0..T-1, negative lat/cost/queue;
 *         the old table is kept), HIP, OOM.
 */
int infaas_sel_load_variants(infaas_sel_t *h, int32_t V,
                             const int32_t *task_id, const int32_t *acc_bp,
                             const int32_t *lat_us, const int32_t *cost,
                             const int32_t *queue_us);

/*
 * Apply a load report (what the workers' monitoring daemons push every few seconds,
 * Section 5): queue_us[d_variant_idx[i]] = d_queue_us[i] for i in 0..n-1.
 *   d_variant_idx [n] DEVICE, rows of the loaded table; must not repeat within one call
 *   d_queue_us    [n] DEVICE, new delay, >= 0
 * An entry whose row is outside 0..V-1 or whose value is negative is skipped.
 * Enqueues on hip_stream (a hipStream_t, NULL = the null stream) and returns.
 * Errors: INVALID_ARG, NOT_LOADED, HIP.
 */
int infaas_sel_update_load(infaas_sel_t *h, int32_t n,
                           const int32_t *d_variant_idx, const int32_t *d_queue_us,
                           void *hip_stream);

/*
 * Decide N queries (Section 4.1).  All arrays are DEVICE memory, structure-of-arrays:
 *   d_task, d_slo_us, d_min_acc_bp, d_batch_idx  [N]  inputs, read only
 *   d_out_variant                                [N]  row of the chosen variant, or -1
 * Results are in the caller's query order.  Enqueues on hip_stream and returns; the call
 * never synchronises the device unless it has to grow its scratch memory (avoid that with
 * infaas_sel_reserve).  N = 0 is a no-op.
 * Errors: INVALID_ARG, NOT_LOADED, HIP, OOM.
 */
int infaas_sel_select(infaas_sel_t *h, int64_t N,
                      const int32_t *d_task, const int32_t *d_slo_us,
                      const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                      int32_t *d_out_variant, void *hip_stream);

/*
 * infaas_sel_select for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results.  It calls
 * no allocating routine, not even on its first use: the one scratch buffer of the lookup kernel
 * (the queues in which its wavefronts park the queries their first probe cannot decide) is a
 * static device array of 20 MiB inside the library, which every GPU the library runs on holds
 * from the moment the library's code is loaded there until the process ends; its address is
 * looked up in infaas_sel_create.  Limits: at most INFAAS_SEL_NOALLOC_MAX_QUERIES queries per
 * call (more: INVALID_ARG; split the batch), a device with at most 256 compute units, and a
 * handle that answers through the staircase index (not INFAAS_SEL_ENGINE_SCAN, whose bucketing
 * needs 20 bytes of scratch per query).  After infaas_sel_load_states it answers from the Active
 * variants only, like infaas_sel_select.  Kernel timing (infaas_sel_set_timing) does not cover it.
 * All calls on one GPU share the array, whichever handle or stream they use: calls that
 * overlap in time on one GPU race and give wrong answers; order them (one stream, or events).
 * Nothing in the array has to survive from call to call and nothing in it needs clearing.
 * Errors: INVALID_ARG (also the limits above; infaas_sel_last_error() says which), NOT_LOADED, HIP.
 */
#define INFAAS_SEL_NOALLOC_MAX_QUERIES ((int64_t)1 << 28)
int infaas_sel_select_noalloc(infaas_sel_t *h, int64_t N,
                              const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, void *hip_stream);

/*
 * infaas_sel_select plus a suggestion for the queries that nothing satisfies: the last step
 * of Section 4.1's Case I, where a variant that comes closest to the accuracy and/or latency
 * target is proposed when no registered variant meets the requirements.  The paper names no
 * distance; this library orders the variants of the query's task (at its batch index) by
 *     1. the number of the two requirements they miss,
 *     2. lat_us[v][b] + queue_us[v] - slo_us where positive, else 0,
 *     3. min_acc_bp - acc_bp[v] where positive, else 0,
 *     4. (cost[v][b], lat_us[v][b], v),
 * exact differences, and takes the first.  Hence, if some variant is within the latency bound,
 * the most accurate of those; else if some variant is accurate enough, the fastest of those;
 * else the fastest of all (the most accurate among equally fast ones).
 *   d_out_variant  [N]  as infaas_sel_select
 *   d_out_closest  [N]  d_out_variant where that is not -1, else the suggestion; -1 only when
 *                       the task has no variants (task or batch index outside the table included)
 * Both DEVICE memory.  On a handle without the staircase index (INFAAS_SEL_ENGINE_SCAN, or a
 * table too large for the index) the suggestions come from an exhaustive pass over the slices
 * of the queries without a selection, behind the scan engine's selection.  A handle with
 * variant states gets INVALID_ARG (infaas_sel_select_tiered_closest is the call for it).
 * Otherwise as infaas_sel_select.
 */
int infaas_sel_select_closest(infaas_sel_t *h, int64_t N,
                              const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, int32_t *d_out_closest, void *hip_stream);

/*
 * ---- State-aware selection: the complete Case I of Section 4.1 ------------------------------
 *
 * Section 4 tracks every variant in a state machine: Inactive (registered, not loaded), Active
 * (loaded, below its peak throughput), Overloaded (at its peak) and Interfered (slower than
 * profiled).  Case I first looks for a match among the Active variants, which incur no loading
 * latency; only if there is none it turns to the Inactive ones and takes the one with the lowest
 * combined loading and inference latency that matches the requirements; Overloaded and
 * Interfered variants are avoided ("Mitigating performance degradation").  Readings where the
 * text is silent: among several Active matches the cheapest, by infaas_sel_select's key; for
 * an Inactive variant the latency requirement is load_us[v] + lat_us[v][b] <= slo_us (no
 * queue: it is not loaded) and the order is (load_us + lat_us[b], lat_us[b], v).
 */
enum { INFAAS_SEL_STATE_INACTIVE = 0, INFAAS_SEL_STATE_ACTIVE = 1,
       INFAAS_SEL_STATE_OVERLOADED = 2, INFAAS_SEL_STATE_INTERFERED = 3 };

/*
 * Give the loaded table its dynamic state.  HOST arrays, copied:
 *   state   [V]  INFAAS_SEL_STATE_*
 *   load_us [V]  loading latency, >= 0, with load_us[v] + lat_us[v][b] <= INT32_MAX
 * Synchronous.  Needs the staircase index (not INFAAS_SEL_ENGINE_SCAN).  From here on
 * infaas_sel_select answers from the Active variants only, infaas_sel_select_closest is not
 * available (infaas_sel_select_tiered_closest takes its place), and infaas_sel_update_load keeps acting on queue_us (which only the Active tier
 * reads).  A later infaas_sel_load_variants drops the states again.
 * Errors: INVALID_ARG, NOT_LOADED, OUT_OF_RANGE (the table stays as it was), HIP, OOM (the table is
 *         dropped: load it again).
 */
int infaas_sel_load_states(infaas_sel_t *h, const int32_t *state, const int32_t *load_us);

/*
 * State report of the monitoring daemons: state[d_variant_idx[i]] = d_state[i] for i < n.
 * Both arrays are DEVICE memory; the rows must be distinct; an entry whose row is outside
 * 0..V-1 or whose code is outside 0..3 is skipped.  Enqueues on hip_stream and returns.
 * Errors: INVALID_ARG, NOT_LOADED (no states loaded), HIP.
 */
int infaas_sel_update_state(infaas_sel_t *h, int32_t n, const int32_t *d_variant_idx,
                            const int32_t *d_state, void *hip_stream);

/*
 * Decide N queries by the two-tier policy above.  Arrays as for infaas_sel_select, plus
 *   d_out_tier  [N]  DEVICE: 1 = the answer is an Active variant, 2 = an Inactive one,
 *                    0 = none (d_out_variant = -1)
 * Keeps 16 bytes of device memory per query of the largest call so far (at most 2^26 queries'
 * worth; longer calls run in passes) for the queries the Active tier leaves open; it is
 * allocated on the first call that needs more, or ahead of time by infaas_sel_reserve.
 * Errors: INVALID_ARG, NOT_LOADED (no states loaded), HIP, OOM.
 */
int infaas_sel_select_tiered(infaas_sel_t *h, int64_t N,
                             const int32_t *d_task, const int32_t *d_slo_us,
                             const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                             int32_t *d_out_variant, int32_t *d_out_tier, void *hip_stream);

/*
 * The complete Case I of Section 4.1 in one call: infaas_sel_select_tiered, and for the queries
 * that no Active and no Inactive variant matches the suggestion the policy ends with -- a variant
 * that comes closest to the accuracy and/or latency target.  Readings, on top of those of
 * infaas_sel_select_closest and infaas_sel_select_tiered: only variants the policy may select are
 * suggested (Active and Inactive, never Overloaded or Interfered); an Active variant is measured
 * by lat_us + queue_us, an Inactive one by load_us + lat_us; the order is (requirements missed,
 * latency beyond slo_us, accuracy below min_acc_bp), then an Active variant before an Inactive
 * one, then the order of the variant's tier.
 *   d_out_closest  [N]  DEVICE: d_out_variant where that is not -1, else the suggestion; -1 only
 *                       when the task has no Active or Inactive variant (task or batch index
 *                       outside the table included)
 * Otherwise as infaas_sel_select_tiered; the device memory kept for the queries the Active tier
 * leaves open is 32 bytes per query of the largest call here (beside each of them goes what the
 * Active tier suggests and how far that is from the requirements).
 */
int infaas_sel_select_tiered_closest(infaas_sel_t *h, int64_t N,
                                     const int32_t *d_task, const int32_t *d_slo_us,
                                     const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                                     int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_closest,
                                     void *hip_stream);

/*
 * ---- Worker selection: the second output of Case I (Section 4.1) ------------------------------
 *
 * The policy returns the variant and the worker that serves the query: for an Active variant
 * the least-loaded worker running an instance of it, for an Inactive one the worker with the
 * lowest utilisation among those that have the variant's target hardware.  A running instance
 * is a {variant, worker} pair (Section 5) with a load figure of its own.  Readings where the
 * text is silent: "least loaded" compares the load figures of the variant's instances, equal
 * ones go to the lower worker number; equal utilisations go to the lower worker number; an
 * Active variant without an instance, or an Inactive one whose hardware no worker has, gets
 * worker -1 while variant and tier stand.
 *
 * Register the cluster.  HOST arrays, copied:
 *   worker_hw    [num_workers]    hardware code of every worker (any int32; compared for equality)
 *   worker_util  [num_workers]    utilisation, >= 0 (e.g. basis points)
 *   variant_hw   [V]              target hardware code of every variant, caller row order
 *   inst_variant [num_instances]  row of the variant the instance runs, 0..V-1
 *   inst_worker  [num_instances]  worker it runs on, 0..num_workers-1
 *   inst_load    [num_instances]  its load, >= 0
 * Synchronous.  Needs infaas_sel_load_states first; a later infaas_sel_load_states or
 * infaas_sel_load_variants drops the cluster again.
 * Errors: INVALID_ARG, NOT_LOADED, OUT_OF_RANGE, HIP, OOM.
 */
int infaas_sel_load_workers(infaas_sel_t *h, int32_t num_workers, const int32_t *worker_hw,
                            const int32_t *worker_util, const int32_t *variant_hw,
                            int32_t num_instances, const int32_t *inst_variant,
                            const int32_t *inst_worker, const int32_t *inst_load);

/*
 * Report of the monitoring daemons: worker_util[d_worker_idx[i]] = d_worker_util[i] for i < n
 * and inst_load[d_inst_idx[j]] = d_inst_load[j] for j < m (instances numbered as they were
 * passed to infaas_sel_load_workers).  DEVICE arrays; either part may be empty (count 0, null
 * pointers); the indices of a part must be distinct; an entry whose index is outside its table
 * or whose value is negative is skipped.  Enqueues on hip_stream and returns.
 * Errors: INVALID_ARG, NOT_LOADED (no workers loaded), HIP.
 */
int infaas_sel_update_workers(infaas_sel_t *h, int32_t n, const int32_t *d_worker_idx,
                              const int32_t *d_worker_util, int32_t m, const int32_t *d_inst_idx,
                              const int32_t *d_inst_load, void *hip_stream);

/*
 * State per running instance.  Section 4 keeps the state machine per variant INSTANCE (the
 * monitoring daemon of the worker that runs it maintains it): a loaded instance is Active,
 * Overloaded or Interfered, a variant that runs nowhere is Inactive.  With instance states the
 * state of a variant is no longer given but follows from its instances: Inactive without any,
 * Active when at least one instance is Active, else Overloaded when some instance is, else
 * Interfered; and the worker of an Active variant is the least-loaded one among those that run
 * an ACTIVE instance of it -- an Overloaded or Interfered instance is avoided while another
 * instance of the same variant serves.  Everything else is as above.
 *   inst_state  [num_instances]  HOST: INFAAS_SEL_STATE_ACTIVE, _OVERLOADED or _INTERFERED, for the
 *                                instances in the order they were passed to infaas_sel_load_workers
 * Synchronous; the states of the variants are replaced by the derived ones.  From here on
 * infaas_sel_update_state is refused (INVALID_ARG): a variant's state changes through its
 * instances.  A later infaas_sel_load_workers drops the instance states (the variants keep the
 * states they had at that moment).
 * Errors: INVALID_ARG, NOT_LOADED (no workers loaded), OUT_OF_RANGE, HIP, OOM.
 */
int infaas_sel_load_instance_states(infaas_sel_t *h, const int32_t *inst_state);

/*
 * Instance state report: the state of instance d_inst_idx[i] becomes d_state[i], i < n.  DEVICE
 * arrays; the indices must be distinct; an entry whose index is outside the table or whose code is
 * not Active, Overloaded or Interfered is skipped.  Enqueues on hip_stream and returns: the
 * report, the states of all variants derived anew, and the rebuild of both tiers' indexes.
 * Errors: INVALID_ARG, NOT_LOADED (no instance states loaded), HIP.
 */
int infaas_sel_update_instance_states(infaas_sel_t *h, int32_t n, const int32_t *d_inst_idx,
                                      const int32_t *d_state, void *hip_stream);

/*
 * infaas_sel_select_tiered plus the worker: arrays as there, and
 *   d_out_worker  [N]  DEVICE: the worker that serves d_out_variant, or -1 (no variant, or no
 *                      worker for it, see above)
 * The first call after a report (of load, state or workers) also enqueues the small kernels
 * that bring the per-variant workers up to date: a caller who captures this call into a HIP
 * graph has to capture the reports with it, or capture again after a report.
 * Errors: INVALID_ARG, NOT_LOADED (no states or no workers loaded), HIP, OOM.
 */
int infaas_sel_select_workers(infaas_sel_t *h, int64_t N,
                              const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_worker,
                              void *hip_stream);

/*
 * The whole of Case I (Section 4.1) in one call: infaas_sel_select_workers and, for the queries
 * neither tier answers, the suggestion of infaas_sel_select_tiered_closest.
 *   d_out_variant, d_out_tier, d_out_worker  [N]  as infaas_sel_select_workers
 *   d_out_closest                            [N]  as infaas_sel_select_tiered_closest (a suggestion
 *                                                 is not served: its d_out_worker stays -1)
 * With instance states loaded the variants' states are the derived ones, as in both calls.
 * Scratch: 32 bytes per query, as infaas_sel_select_tiered_closest.
 * Errors: INVALID_ARG, NOT_LOADED (no states or no workers loaded), HIP, OOM.
 */
int infaas_sel_select_workers_closest(infaas_sel_t *h, int64_t N,
                                      const int32_t *d_task, const int32_t *d_slo_us,
                                      const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                                      int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_worker,
                                      int32_t *d_out_closest, void *hip_stream);

/*
 * ---- Scaling decision on a change in query load: Case II, scaling up (Section 4.2.2) ----------
 *
 * For a running variant cur with n_cur instances and an incoming load of L queries per second:
 * nothing, when Q[cur] * n_cur already carries slack_pct percent of L (constraint 1 of the
 * integer program of Section 4.2.1; the paper's slack-threshold 1.05 is 105); else either
 * REPLICATE, load inst(cur) - n_cur more instances of cur, allowed when lat_us[cur][b] <= slo_us
 * (constraint 2 binds every newly loaded instance), or UPGRADE, load inst(u) instances of a
 * variant u of the same model architecture with lat_us[u][b] <= slo_us and Q[u] > Q[cur] and
 * unload cur -- where inst(v) = ceil(L * slack_pct / (100 * Q[v])).  The cheaper one by the
 * program's objective wins:
 *     replicate:  C[cur] * (inst(cur) - n_cur) * (1 + lambda * T_load[cur])
 *     upgrade:    C[u] * inst(u) * (1 + lambda * T_load[u]) - C[cur] * n_cur
 * in exact integer arithmetic (lambda per second, T_load in microseconds, 128-bit products).
 * Readings where the text is silent: among upgrades of equal cost the lower row; replication
 * wins a tie against the cheapest upgrade; worker resources (constraint 3) are not part of the
 * decision.  Scaling down is infaas_sel_scale_down.
 *
 * Register what the decision reads per variant.  HOST arrays [V], caller row order, copied:
 *   arch_id   model architecture (any int32; compared for equality)
 *   sat_qps   saturation throughput Q in queries per second, >= 1
 *   hw_cost   hardware cost C per second, 0..1,048,576
 *   load_us   loading latency T_load, >= 0
 * and lambda_per_s in 0..1000, slack_pct in 0..200.  Synchronous.  Independent of
 * infaas_sel_load_states / _load_workers; a later infaas_sel_load_variants drops it.
 * Errors: INVALID_ARG, NOT_LOADED, OUT_OF_RANGE, HIP, OOM.
 */
int infaas_sel_load_scaling(infaas_sel_t *h, const int32_t *arch_id, const int32_t *sat_qps,
                            const int32_t *hw_cost, const int32_t *load_us,
                            int32_t lambda_per_s, int32_t slack_pct);

/*
 * Decide R requests.  DEVICE arrays [R]:
 *   d_variant, d_instances, d_load_qps, d_slo_us, d_batch_idx   the running variant (row), its
 *       running instances (0..1,000,000), the incoming load (0..1,000,000,000), the latency
 *       objective and the batch-size index; a request outside these ranges gets no action
 *   d_out_action     0 nothing to do, 1 replicate, 2 upgrade, 3 scaling needed but neither
 *                    option is allowed (the worker has to turn to the controller)
 *   d_out_variant    the variant to load (the running one for 1), -1 for actions 0 and 3
 *   d_out_instances  instances of it to load, 0 for actions 0 and 3
 * Enqueues on hip_stream and returns; allocates nothing.
 * Errors: INVALID_ARG, NOT_LOADED (no scaling profile loaded), HIP.
 */
int infaas_sel_scale(infaas_sel_t *h, int64_t R,
                     const int32_t *d_variant, const int32_t *d_instances, const int32_t *d_load_qps,
                     const int32_t *d_slo_us, const int32_t *d_batch_idx,
                     int32_t *d_out_action, int32_t *d_out_variant, int32_t *d_out_instances,
                     void *hip_stream);

/*
 * ---- Scaling down (Section 4.2.2, "Scaling down algorithm") ------------------------------------
 *
 * Asked at regular intervals: can the incoming load L of the running variant cur with n_cur
 * instances be carried for less?  Either REMOVE one instance of cur, allowed when at least one
 * stays and Q[cur] * (n_cur - 1) carries slack_pct percent of L; or DOWNGRADE to a variant u of the
 * same model architecture with a lower hardware cost, C[u] < C[cur], and lat_us[u][b] <= slo_us:
 * load inst(u) = max(1, ceil(L * slack_pct / (100 * Q[u]))) instances of u and unload cur.  By the
 * objective of the integer program, as in infaas_sel_scale:
 *     keep:       0
 *     remove:     - C[cur]
 *     downgrade:  C[u] * inst(u) * (1 + lambda * T_load[u]) - C[cur] * n_cur
 * the lowest wins, and only an option that lowers the objective is acted on.  Readings where the
 * text is silent: one instance per decision, never the last one (unloading a variant altogether
 * belongs to the state machine of Section 4); ties go to keeping, then to removing, then to the
 * lower row.  The paper has the autoscaler wait T_v = T_load[cur] before it executes the action;
 * that wait is the caller's and does not enter the decision.
 *
 * Uses what infaas_sel_load_scaling registered.  DEVICE arrays [R], requests as for
 * infaas_sel_scale (same ranges; a request outside them gets action 0), and
 *   d_out_action     0 keep, 1 remove, 2 downgrade
 *   d_out_variant    cur for 1, u for 2, -1 for 0
 *   d_out_instances  1 instance to unload for 1; inst(u) instances to load for 2 (all n_cur of cur
 *                    are then unloaded); 0 for 0
 * Enqueues on hip_stream and returns; allocates nothing.
 * Errors: INVALID_ARG, NOT_LOADED (no scaling profile loaded), HIP.
 */
int infaas_sel_scale_down(infaas_sel_t *h, int64_t R,
                          const int32_t *d_variant, const int32_t *d_instances, const int32_t *d_load_qps,
                          const int32_t *d_slo_us, const int32_t *d_batch_idx,
                          int32_t *d_out_action, int32_t *d_out_variant, int32_t *d_out_instances,
                          void *hip_stream);

/* Free the handle and everything it owns.  NULL is a no-op. */
void infaas_sel_destroy(infaas_sel_t *h);

/* ---- helpers around the calls above ------------------------------------------- */

/* Pre-grow the scratch memory for calls of up to max_queries queries, so that
 * infaas_sel_select (with states loaded: infaas_sel_select_tiered) does not allocate.
 * Errors: INVALID_ARG, HIP, OOM. */
int infaas_sel_reserve(infaas_sel_t *h, int64_t max_queries);

/* Copy the current queue_us back to HOST memory [V], in the caller's row order, after
 * synchronising hip_stream.  For tests of infaas_sel_update_load. */
int infaas_sel_read_load(infaas_sel_t *h, int32_t *queue_us, void *hip_stream);

/* Per-kernel timing.  When enabled, every kernel the library launches is bracketed by HIP
 * events on the caller's stream; infaas_sel_get_timings synchronises those events and
 * returns, per kernel, the number of launches and the summed duration since the last
 * reset.  Kernel ids are INFAAS_SEL_K_*. */
enum {
    INFAAS_SEL_K_UPDATE = 0,     /* load-update scatter */
    INFAAS_SEL_K_HISTOGRAM = 1,  /* scan engine: queries per slice */
    INFAAS_SEL_K_PLAN = 2,       /* scan engine: prefix sums and tile plan */
    INFAAS_SEL_K_SCATTER = 3,    /* scan engine: bucket the queries */
    INFAAS_SEL_K_SCAN_LDS = 4,   /* scan engine: LDS-staged filter + argmin */
    INFAAS_SEL_K_SCAN_WIDE = 5,  /* scan engine: device-wide path for large slices */
    INFAAS_SEL_K_FINISH_WIDE = 6,/* scan engine: decode the device-wide minima */
    INFAAS_SEL_K_INDEX_BUILD = 7,/* staircase index (re)build */
    INFAAS_SEL_K_INDEX_SELECT = 8,/* staircase index lookup, one lane per query */
    INFAAS_SEL_K_UPDATE_STATE = 9,/* state report: masks of the rank-ordered columns */
    INFAAS_SEL_K_WORKER_REPORT = 10,/* utilisation and instance-load report */
    INFAAS_SEL_K_WORKER_TABLES = 11,/* worker of every variant (two kernels) */
    INFAAS_SEL_K_STEP_WORKERS = 12,/* worker of every step of an index */
    INFAAS_SEL_K_SCALE = 13,     /* scaling decisions */
    INFAAS_SEL_K_GROUP_BIN = 14, /* grouped index: queries binned by group of tasks */
    INFAAS_SEL_K_GROUP_LOOKUP = 15,/* grouped index: lookup, one group's bodies in LDS per workgroup */
    INFAAS_SEL_K_GROUP_FINISH = 16,/* grouped index: answers back into query order */
    INFAAS_SEL_K_INSTANCE_STATES = 17,/* instance state report and the variants' states derived from it */
    INFAAS_SEL_K_CLOSEST_SCAN = 18,/* closest-variant suggestions by exhaustive scan (no index) */
    INFAAS_SEL_K_SCALE_DOWN = 19,/* scaling-down decisions */
    INFAAS_SEL_K_COUNT = 20
};
typedef struct {
    int64_t launches[INFAAS_SEL_K_COUNT];
    double total_ms[INFAAS_SEL_K_COUNT];
} infaas_sel_timings;
int infaas_sel_set_timing(infaas_sel_t *h, int32_t enabled); /* also resets the counters */
int infaas_sel_get_timings(infaas_sel_t *h, infaas_sel_timings *out);

/* Sizes the library derived from the loaded table. */
typedef struct {
    int32_t num_variants;       /* V */
    int32_t num_slices;         /* T*B */
    int32_t max_segment;        /* most variants in one task */
    int32_t lds_segment_limit;  /* effective value */
    int32_t wide_segments;      /* tasks handled by the device-wide scan path */
    int32_t index_in_lds;       /* 1 when the lookup kernel mirrors the index in LDS (all of it, or
                                   as many slices as fit; the others are read from global memory) */
    int32_t index_truncated;    /* slices whose staircase was cut at its capacity or not stored */
    int32_t index_max_steps;    /* longest staircase of any slice (as stored) */
    int32_t index_hot_rows;     /* steps per slice whose caller row is kept beside the index in LDS */
    int64_t index_bytes;        /* size of the staircase index (as of the latest build a selection has run behind) */
    int64_t index_steps;        /* steps over all slices */
    int64_t table_bytes;        /* device bytes of the variant store */
    int64_t scratch_bytes;      /* device bytes of scratch currently reserved */
    /* The most recent launch of the index lookup kernel on this handle (for a state-aware call: the
     * Inactive tier's): the queries whose answer the first group of their slice's staircase, as
     * mirrored in LDS, could not decide, and what became of them.  Valid once the caller has
     * synchronised the stream of that call; infaas_sel_get_info copies them with a blocking hipMemcpy. */
    int64_t lookup_parked;      /* queries set aside for the slower paths */
    int64_t lookup_second_body; /* ... answered by the second group of steps */
    int64_t lookup_global_body; /* ... answered by a first group read from global memory (slice not in LDS) */
    int64_t lookup_scanned;     /* ... sent through the rank-ordered scan of the slice */
    int64_t lookup_unanswered;  /* ... that ended without a feasible variant */
    int32_t index_groups;       /* 1: one LDS holds (part of) the whole index; more: the tasks are dealt to this many
                                   groups whose staircases fit one LDS each, and calls of a million queries or more
                                   are binned by group and looked up group by group */
    int32_t reserved0;
} infaas_sel_info;
int infaas_sel_get_info(infaas_sel_t *h, infaas_sel_info *out);

/* Static text for a status code. */
const char *infaas_sel_strerror(int status);

/* Text of the HIP call that failed most recently on the calling thread (which call, HIP's
 * message); empty if none has.  Valid until the next failure on that thread. */
const char *infaas_sel_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* INFAAS_SEL_H */
