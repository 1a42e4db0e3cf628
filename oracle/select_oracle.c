/*
 * CPU oracle for per-query model-variant selection (INFaaS, arxiv 1905.13348).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * selection computes.  It exists so that tests, the smoke check and the
 * benchmark's CPU-baseline leg have something to compare the GPU library with.
 * The product library never links, loads or calls it, and it shares no code,
 * header, table or helper with the GPU path.
 *
 * What is computed (Section 4.1, "Case I: on arrival of a query"; cheapest-choice
 * objective as in the worked example of Section 2.2, Tables 2 and 3):
 *
 *   A query names a task (application), a latency objective slo_us, a minimum
 *   accuracy min_acc_bp and a batch-size index b.  Among the registered variants
 *   of that task, a variant v is FEASIBLE when
 *       acc_bp[v] >= min_acc_bp                          (accuracy requirement)
 *       lat_us[v][b] + queue_us[v] <= slo_us             (latency requirement;
 *                                   "<=" as in the autoscaler's SLO constraint
 *                                   T_inf <= S of Section 4.2; queue_us is the
 *                                   dynamic state that Section 4 says must be
 *                                   taken into account besides the static
 *                                   profile)
 *   and the answer is the feasible variant with the lexicographically smallest
 *       (cost[v][b], lat_us[v][b], v)
 *   i.e. the cheapest one, ties broken by profiled latency and then by the
 *   caller's row index.  If no variant is feasible the answer is -1 (the
 *   "no registered variant can meet the requirements" outcome of Section 4.1).
 *
 *   The brute-force search over all variants is the yardstick the paper itself
 *   uses (Section 6.4), so the oracle IS that search: no sorting, no index, no
 *   packing of keys.
 *
 * Readings taken where the paper is silent:
 *   - the sum lat+queue is formed in 64 bits, so it cannot wrap;
 *   - a task id or batch index outside the table, or a task with no variants,
 *     has an empty feasible set, hence -1;
 *   - load updates are applied in array order; an update whose row is outside
 *     0..V-1 or whose value is negative is skipped.
 *
 * Pins (tests/, "not gpu"): the printed example of Tables 2/3, an independent
 * numpy enumerator on tiny tables, invariants (chosen variant feasible, nothing
 * feasible is smaller, -1 iff nothing feasible), special cases that reduce to a
 * lexicographic sort, monotonicity and shift invariance, and seeded mutants of
 * this file that each pin set must reject.  The closest-variant search further
 * down follows a reading of this file's own (the paper names no distance); it is
 * pinned by two independently written numpy enumerators (one by cases, one by a
 * sorted key), structural properties, extreme values and its own mutants.  The
 * state-aware selection at the end follows Sections 4 and 4.1 with the readings
 * listed there; it is pinned by a numpy enumerator, by two special cases that
 * reduce to the plain selection (all variants Active; all Inactive), by hand-built
 * policy cases and by twelve mutants.  The worker selection behind it (the second
 * output of Case I) is pinned by a numpy enumerator, by hand-built cases (one
 * instance, one hardware class, ties, no instance, no worker of the hardware),
 * by invariance under reordering of the instance list and by its own mutants.
 * The scaling decision (last routine) is pinned by the instance counts and costs
 * the paper prints in Tables 2 and 3, by an enumerator in Python's unbounded
 * integers, by closed forms (lambda = 0: the hardware cost of the resulting
 * configuration decides) and by its own mutants.
 * The only statement that stays
 * "parity unpinned" is the count of valid options printed in Table 7, because
 * the profiles behind it are not published.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* 1 when variant row v is feasible for the query (slo, min_acc, b). */
static int feasible(const int32_t *acc_bp, const int32_t *lat_us, const int32_t *queue_us,
                    int32_t B, int64_t v, int32_t slo_us, int32_t min_acc_bp, int32_t b)
{
    if (acc_bp[v] < min_acc_bp)
        return 0;
    int64_t total = (int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];
    if (total > (int64_t)slo_us)
        return 0;
    return 1;
}

/* 1 when (cost, lat, row) of v is lexicographically smaller than that of w. */
static int cheaper(const int32_t *lat_us, const int32_t *cost, int32_t B, int32_t b,
                   int64_t v, int64_t w)
{
    int32_t cv = cost[v * B + b], cw = cost[w * B + b];
    if (cv != cw)
        return cv < cw;
    int32_t lv = lat_us[v * B + b], lw = lat_us[w * B + b];
    if (lv != lw)
        return lv < lw;
    return v < w;
}

/*
 * Literal form: every query looks at every row of the table, in the caller's
 * order.  O(N*V); meant for small tables and as the cross-check of the grouped
 * form below.  Returns 0, or -1 on bad arguments.
 */
int oracle_select_literal(int64_t V, int32_t B,
                          const int32_t *task_id, const int32_t *acc_bp,
                          const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                          int64_t N,
                          const int32_t *q_task, const int32_t *q_slo_us,
                          const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                          int32_t *out_variant)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    for (int64_t q = 0; q < N; ++q) {
        int64_t best = -1;
        int32_t b = q_batch_idx[q];
        if (b >= 0 && b < B) {
            for (int64_t v = 0; v < V; ++v) {
                if (task_id[v] != q_task[q])
                    continue;
                if (!feasible(acc_bp, lat_us, queue_us, B, v, q_slo_us[q], q_min_acc_bp[q], b))
                    continue;
                if (best < 0 || cheaper(lat_us, cost, B, b, v, best))
                    best = v;
            }
        }
        out_variant[q] = (int32_t)best;
    }
    return 0;
}

/*
 * Grouped form: the rows of each task are listed once (in the caller's order),
 * then every query runs the same brute-force search over its task's list only.
 * Same result as the literal form; O(N * variants-per-task).  Queries are
 * independent, so the outer loop may run on several host threads.
 */
int oracle_select(int64_t V, int32_t B,
                  const int32_t *task_id, const int32_t *acc_bp,
                  const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                  int64_t N,
                  const int32_t *q_task, const int32_t *q_slo_us,
                  const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                  int32_t *out_variant)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t T = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (task_id[v] < 0)
            return -1;
        if ((int64_t)task_id[v] + 1 > T)
            T = (int64_t)task_id[v] + 1;
    }
    int64_t *first = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    int64_t *fill = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    if (!first || !rows || !fill) {
        free(first); free(rows); free(fill);
        return -1;
    }
    for (int64_t v = 0; v < V; ++v)
        first[task_id[v] + 1] += 1;
    for (int64_t t = 0; t < T; ++t)
        first[t + 1] += first[t];
    for (int64_t v = 0; v < V; ++v) {
        int64_t t = task_id[v];
        rows[first[t] + fill[t]] = v;
        fill[t] += 1;
    }

#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int64_t best = -1;
        int32_t b = q_batch_idx[q];
        int64_t t = q_task[q];
        if (b >= 0 && b < B && t >= 0 && t < T) {
            for (int64_t i = first[t]; i < first[t + 1]; ++i) {
                int64_t v = rows[i];
                if (!feasible(acc_bp, lat_us, queue_us, B, v, q_slo_us[q], q_min_acc_bp[q], b))
                    continue;
                if (best < 0 || cheaper(lat_us, cost, B, b, v, best))
                    best = v;
            }
        }
        out_variant[q] = (int32_t)best;
    }
    free(first); free(rows); free(fill);
    return 0;
}

/*
 * Size of the feasible set of each query (the "valid options" column of the
 * decision-overhead table in Section 6.4).  Diagnostic; literal scan.
 */
int oracle_count_feasible(int64_t V, int32_t B,
                          const int32_t *task_id, const int32_t *acc_bp,
                          const int32_t *lat_us, const int32_t *queue_us,
                          int64_t N,
                          const int32_t *q_task, const int32_t *q_slo_us,
                          const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                          int32_t *out_count)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    for (int64_t q = 0; q < N; ++q) {
        int32_t n = 0;
        int32_t b = q_batch_idx[q];
        if (b >= 0 && b < B)
            for (int64_t v = 0; v < V; ++v)
                if (task_id[v] == q_task[q] &&
                    feasible(acc_bp, lat_us, queue_us, B, v, q_slo_us[q], q_min_acc_bp[q], b))
                    n += 1;
        out_count[q] = n;
    }
    return 0;
}

/*
 * Load update (the monitoring daemons' periodic push of per-variant load,
 * Section 5): queue_us[row[i]] = value[i], in array order.
 */
void oracle_update_load(int64_t V, int32_t *queue_us, int64_t n,
                        const int32_t *variant_idx, const int32_t *new_queue_us)
{
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = variant_idx[i];
        if (v < 0 || v >= V || new_queue_us[i] < 0)
            continue;
        queue_us[v] = new_queue_us[i];
    }
}

/*
 * Closest variant (Section 4.1, last step of Case I): when no registered variant
 * meets the requirements, a variant that comes closest to the accuracy and/or
 * latency target is suggested.  The paper names no distance.  The reading taken
 * here orders the variants of the task by, in this order,
 *     1. how many of the two requirements they miss (0, 1 or 2),
 *     2. by how much lat_us[v][b] + queue_us[v] exceeds slo_us (0 when it fits),
 *     3. by how much acc_bp[v] falls short of min_acc_bp (0 when it meets it),
 *     4. the selection key (cost[v][b], lat_us[v][b], v),
 * all differences formed in 64 bits, and suggests the first one.  A variant that
 * meets both requirements has (0, 0, 0) in front of its key, so for a query with
 * a non-empty feasible set the suggestion IS the selected variant.  The result is
 * -1 only when the task has no variants at that batch index (task or batch index
 * outside the table included).
 */
typedef struct {
    int missed;          /* requirements not met */
    int64_t over_us;     /* latency beyond the objective */
    int64_t short_bp;    /* accuracy below the minimum */
} distance_t;

static distance_t distance_of(const int32_t *acc_bp, const int32_t *lat_us, const int32_t *queue_us,
                              int32_t B, int64_t v, int32_t slo_us, int32_t min_acc_bp, int32_t b)
{
    distance_t d;
    int64_t total = (int64_t)lat_us[v * B + b] + (int64_t)queue_us[v];
    d.over_us = total > (int64_t)slo_us ? total - (int64_t)slo_us : 0;
    d.short_bp = acc_bp[v] < min_acc_bp ? (int64_t)min_acc_bp - (int64_t)acc_bp[v] : 0;
    d.missed = (d.over_us > 0) + (d.short_bp > 0);
    return d;
}

/* 1 when v comes before w in the order above. */
static int closer(const int32_t *acc_bp, const int32_t *lat_us, const int32_t *cost,
                  const int32_t *queue_us, int32_t B, int32_t slo_us, int32_t min_acc_bp, int32_t b,
                  int64_t v, int64_t w)
{
    distance_t dv = distance_of(acc_bp, lat_us, queue_us, B, v, slo_us, min_acc_bp, b);
    distance_t dw = distance_of(acc_bp, lat_us, queue_us, B, w, slo_us, min_acc_bp, b);
    if (dv.missed != dw.missed)
        return dv.missed < dw.missed;
    if (dv.over_us != dw.over_us)
        return dv.over_us < dw.over_us;
    if (dv.short_bp != dw.short_bp)
        return dv.short_bp < dw.short_bp;
    return cheaper(lat_us, cost, B, b, v, w);
}

/*
 * Literal form: every query looks at every row of the table.  out_variant gets
 * the selection (as oracle_select_literal), out_closest the suggestion.
 */
int oracle_select_closest_literal(int64_t V, int32_t B,
                                  const int32_t *task_id, const int32_t *acc_bp,
                                  const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                                  int64_t N,
                                  const int32_t *q_task, const int32_t *q_slo_us,
                                  const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                                  int32_t *out_variant, int32_t *out_closest)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    for (int64_t q = 0; q < N; ++q) {
        int64_t best = -1;
        int32_t b = q_batch_idx[q];
        if (b >= 0 && b < B) {
            for (int64_t v = 0; v < V; ++v) {
                if (task_id[v] != q_task[q])
                    continue;
                if (best < 0 || closer(acc_bp, lat_us, cost, queue_us, B, q_slo_us[q], q_min_acc_bp[q], b, v, best))
                    best = v;
            }
        }
        out_closest[q] = (int32_t)best;
        out_variant[q] = (best >= 0 && feasible(acc_bp, lat_us, queue_us, B, best, q_slo_us[q], q_min_acc_bp[q], b))
                             ? (int32_t)best : -1;
    }
    return 0;
}

/* Grouped form of the same search (rows listed per task once, queries on several host threads). */
int oracle_select_closest(int64_t V, int32_t B,
                          const int32_t *task_id, const int32_t *acc_bp,
                          const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                          int64_t N,
                          const int32_t *q_task, const int32_t *q_slo_us,
                          const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                          int32_t *out_variant, int32_t *out_closest)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t T = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (task_id[v] < 0)
            return -1;
        if ((int64_t)task_id[v] + 1 > T)
            T = (int64_t)task_id[v] + 1;
    }
    int64_t *first = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    int64_t *fill = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    if (!first || !rows || !fill) {
        free(first); free(rows); free(fill);
        return -1;
    }
    for (int64_t v = 0; v < V; ++v)
        first[task_id[v] + 1] += 1;
    for (int64_t t = 0; t < T; ++t)
        first[t + 1] += first[t];
    for (int64_t v = 0; v < V; ++v) {
        int64_t t = task_id[v];
        rows[first[t] + fill[t]] = v;
        fill[t] += 1;
    }

#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int64_t best = -1;
        int32_t b = q_batch_idx[q];
        int64_t t = q_task[q];
        if (b >= 0 && b < B && t >= 0 && t < T) {
            for (int64_t i = first[t]; i < first[t + 1]; ++i) {
                int64_t v = rows[i];
                if (best < 0 || closer(acc_bp, lat_us, cost, queue_us, B, q_slo_us[q], q_min_acc_bp[q], b, v, best))
                    best = v;
            }
        }
        out_closest[q] = (int32_t)best;
        out_variant[q] = (best >= 0 && feasible(acc_bp, lat_us, queue_us, B, best, q_slo_us[q], q_min_acc_bp[q], b))
                             ? (int32_t)best : -1;
    }
    free(first); free(rows); free(fill);
    return 0;
}

/*
 * State-aware selection (Section 4, "State machine for the lifecycle of model-variants", and
 * the full text of Case I in Section 4.1, plus "Mitigating performance degradation"):
 * every variant is Inactive (registered, not loaded), Active (loaded, below its peak
 * throughput), Overloaded (at its peak) or Interfered (slower than profiled).  The policy
 * first looks among the ACTIVE variants that match the query's requirements, because they
 * incur no loading latency; only if there is none it turns to the INACTIVE ones and takes
 * the one with the lowest combined loading and inference latency that matches the
 * requirements; Overloaded and Interfered variants are avoided.
 *
 * Readings taken where the text is silent:
 *   - tier 1 (Active): requirements as in the plain selection (accuracy, and latency plus
 *     queueing delay within the objective); among several matches the cheapest, by the plain
 *     key (cost, lat, row);
 *   - tier 2 (Inactive): accuracy as before; the latency requirement applies to the combined
 *     latency load_us[v] + lat_us[v][b] (an unloaded variant has no queue); the order is
 *     (load_us + lat_us[b], lat_us[b], row);
 *   - states are coded 0 Inactive, 1 Active, 2 Overloaded, 3 Interfered; any other code is
 *     never selected.
 * out_tier is 1 or 2 for the tier the answer comes from and 0 with out_variant = -1.
 */
enum { STATE_INACTIVE = 0, STATE_ACTIVE = 1, STATE_OVERLOADED = 2, STATE_INTERFERED = 3 };

/* 1 when the unloaded variant v comes before w: lower load + inference latency, then lower
 * inference latency, then lower row. */
static int loads_sooner(const int32_t *lat_us, const int32_t *load_us, int32_t B, int32_t b,
                        int64_t v, int64_t w)
{
    int64_t tv = (int64_t)load_us[v] + (int64_t)lat_us[v * B + b];
    int64_t tw = (int64_t)load_us[w] + (int64_t)lat_us[w * B + b];
    if (tv != tw)
        return tv < tw;
    int32_t run_v = lat_us[v * B + b], run_w = lat_us[w * B + b];
    if (run_v != run_w)
        return run_v < run_w;
    return v < w;
}

/* One query of the state-aware selection against the rows rows[0..n) (all of the query's task). */
static void tiered_one(const int64_t *rows, int64_t n, int32_t B,
                       const int32_t *acc_bp, const int32_t *lat_us, const int32_t *cost,
                       const int32_t *queue_us, const int32_t *state, const int32_t *load_us,
                       int32_t slo_us, int32_t min_acc_bp, int32_t b,
                       int32_t *out_variant, int32_t *out_tier)
{
    int64_t active = -1, inactive = -1;
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = rows[i];
        if (state[v] == STATE_ACTIVE) {
            if (!feasible(acc_bp, lat_us, queue_us, B, v, slo_us, min_acc_bp, b))
                continue;
            if (active < 0 || cheaper(lat_us, cost, B, b, v, active))
                active = v;
        } else if (state[v] == STATE_INACTIVE) {
            if (acc_bp[v] < min_acc_bp)
                continue;
            if ((int64_t)load_us[v] + (int64_t)lat_us[v * B + b] > (int64_t)slo_us)
                continue;
            if (inactive < 0 || loads_sooner(lat_us, load_us, B, b, v, inactive))
                inactive = v;
        }
    }
    *out_variant = (int32_t)(active >= 0 ? active : inactive);
    *out_tier = active >= 0 ? 1 : (inactive >= 0 ? 2 : 0);
}

/* Literal form: every query looks at every row of the table. */
int oracle_select_tiered_literal(int64_t V, int32_t B,
                                 const int32_t *task_id, const int32_t *acc_bp,
                                 const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                                 const int32_t *state, const int32_t *load_us,
                                 int64_t N,
                                 const int32_t *q_task, const int32_t *q_slo_us,
                                 const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                                 int32_t *out_variant, int32_t *out_tier)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    if (!rows)
        return -1;
    for (int64_t q = 0; q < N; ++q) {
        int64_t n = 0;
        int32_t b = q_batch_idx[q];
        if (b >= 0 && b < B)
            for (int64_t v = 0; v < V; ++v)
                if (task_id[v] == q_task[q])
                    rows[n++] = v;
        tiered_one(rows, n, B, acc_bp, lat_us, cost, queue_us, state, load_us, q_slo_us[q],
                   q_min_acc_bp[q], b, &out_variant[q], &out_tier[q]);
    }
    free(rows);
    return 0;
}

/* Grouped form (rows listed per task once, queries on several host threads). */
int oracle_select_tiered(int64_t V, int32_t B,
                         const int32_t *task_id, const int32_t *acc_bp,
                         const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                         const int32_t *state, const int32_t *load_us,
                         int64_t N,
                         const int32_t *q_task, const int32_t *q_slo_us,
                         const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                         int32_t *out_variant, int32_t *out_tier)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t T = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (task_id[v] < 0)
            return -1;
        if ((int64_t)task_id[v] + 1 > T)
            T = (int64_t)task_id[v] + 1;
    }
    int64_t *first = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    int64_t *fill = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    if (!first || !rows || !fill) {
        free(first); free(rows); free(fill);
        return -1;
    }
    for (int64_t v = 0; v < V; ++v)
        first[task_id[v] + 1] += 1;
    for (int64_t t = 0; t < T; ++t)
        first[t + 1] += first[t];
    for (int64_t v = 0; v < V; ++v) {
        int64_t t = task_id[v];
        rows[first[t] + fill[t]] = v;
        fill[t] += 1;
    }
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int32_t b = q_batch_idx[q];
        int64_t t = q_task[q];
        int64_t n = (b >= 0 && b < B && t >= 0 && t < T) ? first[t + 1] - first[t] : 0;
        tiered_one(n ? rows + first[t] : rows, n, B, acc_bp, lat_us, cost, queue_us, state, load_us,
                   q_slo_us[q], q_min_acc_bp[q], b, &out_variant[q], &out_tier[q]);
    }
    free(first); free(rows); free(fill);
    return 0;
}

/*
 * The complete Case I of Section 4.1 in one pass: a match among the Active variants; else a
 * match among the Inactive ones; else -- no registered variant meets the requirements -- the
 * suggestion of the variant that comes closest to the accuracy and/or latency target.
 *
 * Readings taken for the last step, on top of those of the state-aware selection and of the
 * closest-variant suggestion above:
 *   - only variants that the policy may select at all are suggested: Active and Inactive ones,
 *     never Overloaded or Interfered ones;
 *   - the latency a variant is measured by is the one its tier is selected by: lat + queue for
 *     an Active variant, load + lat for an Inactive one;
 *   - the order is (requirements missed, latency beyond the objective, accuracy below the
 *     minimum), exact 64-bit differences; then an Active variant before an Inactive one (it
 *     needs no loading); then the order of the variant's tier -- (cost, lat, row) among Active,
 *     (load + lat, lat, row) among Inactive variants.
 * out_closest is out_variant where a variant was selected, else the suggestion, else -1 (the
 * task has no Active or Inactive variant at that batch index).
 */
static distance_t tier_distance(const int32_t *acc_bp, const int32_t *lat_us, const int32_t *queue_us,
                                const int32_t *state, const int32_t *load_us, int32_t B, int64_t v,
                                int32_t slo_us, int32_t min_acc_bp, int32_t b)
{
    distance_t d;
    int64_t wait = state[v] == STATE_ACTIVE ? (int64_t)queue_us[v] : (int64_t)load_us[v];
    int64_t total = (int64_t)lat_us[v * B + b] + wait;
    d.over_us = total > (int64_t)slo_us ? total - (int64_t)slo_us : 0;
    d.short_bp = acc_bp[v] < min_acc_bp ? (int64_t)min_acc_bp - (int64_t)acc_bp[v] : 0;
    d.missed = (d.over_us > 0) + (d.short_bp > 0);
    return d;
}

/* 1 when v comes before w as a suggestion; both are Active or Inactive. */
static int suggested_before(const int32_t *acc_bp, const int32_t *lat_us, const int32_t *cost,
                            const int32_t *queue_us, const int32_t *state, const int32_t *load_us,
                            int32_t B, int32_t slo_us, int32_t min_acc_bp, int32_t b, int64_t v, int64_t w)
{
    distance_t dv = tier_distance(acc_bp, lat_us, queue_us, state, load_us, B, v, slo_us, min_acc_bp, b);
    distance_t dw = tier_distance(acc_bp, lat_us, queue_us, state, load_us, B, w, slo_us, min_acc_bp, b);
    if (dv.missed != dw.missed)
        return dv.missed < dw.missed;
    if (dv.over_us != dw.over_us)
        return dv.over_us < dw.over_us;
    if (dv.short_bp != dw.short_bp)
        return dv.short_bp < dw.short_bp;
    if (state[v] != state[w])
        return state[v] == STATE_ACTIVE;
    return state[v] == STATE_ACTIVE ? cheaper(lat_us, cost, B, b, v, w) : loads_sooner(lat_us, load_us, B, b, v, w);
}

static void case1_one(const int64_t *rows, int64_t n, int32_t B,
                      const int32_t *acc_bp, const int32_t *lat_us, const int32_t *cost,
                      const int32_t *queue_us, const int32_t *state, const int32_t *load_us,
                      int32_t slo_us, int32_t min_acc_bp, int32_t b,
                      int32_t *out_variant, int32_t *out_tier, int32_t *out_closest)
{
    tiered_one(rows, n, B, acc_bp, lat_us, cost, queue_us, state, load_us, slo_us, min_acc_bp, b,
               out_variant, out_tier);
    if (*out_variant >= 0) {
        *out_closest = *out_variant;
        return;
    }
    int64_t best = -1;
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = rows[i];
        if (state[v] != STATE_ACTIVE && state[v] != STATE_INACTIVE)
            continue;
        if (best < 0 || suggested_before(acc_bp, lat_us, cost, queue_us, state, load_us, B, slo_us,
                                         min_acc_bp, b, v, best))
            best = v;
    }
    *out_closest = (int32_t)best;
}

/* Literal form: every query looks at every row of the table. */
int oracle_select_case1_literal(int64_t V, int32_t B,
                                const int32_t *task_id, const int32_t *acc_bp,
                                const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                                const int32_t *state, const int32_t *load_us,
                                int64_t N,
                                const int32_t *q_task, const int32_t *q_slo_us,
                                const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                                int32_t *out_variant, int32_t *out_tier, int32_t *out_closest)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    if (!rows)
        return -1;
    for (int64_t q = 0; q < N; ++q) {
        int64_t n = 0;
        int32_t b = q_batch_idx[q];
        if (b >= 0 && b < B)
            for (int64_t v = 0; v < V; ++v)
                if (task_id[v] == q_task[q])
                    rows[n++] = v;
        case1_one(rows, n, B, acc_bp, lat_us, cost, queue_us, state, load_us, q_slo_us[q],
                  q_min_acc_bp[q], b, &out_variant[q], &out_tier[q], &out_closest[q]);
    }
    free(rows);
    return 0;
}

/* Grouped form (rows listed per task once, queries on several host threads). */
int oracle_select_case1(int64_t V, int32_t B,
                        const int32_t *task_id, const int32_t *acc_bp,
                        const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                        const int32_t *state, const int32_t *load_us,
                        int64_t N,
                        const int32_t *q_task, const int32_t *q_slo_us,
                        const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                        int32_t *out_variant, int32_t *out_tier, int32_t *out_closest)
{
    if (V < 0 || B <= 0 || N < 0)
        return -1;
    int64_t T = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (task_id[v] < 0)
            return -1;
        if ((int64_t)task_id[v] + 1 > T)
            T = (int64_t)task_id[v] + 1;
    }
    int64_t *first = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * (size_t)(V > 0 ? V : 1));
    int64_t *fill = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    if (!first || !rows || !fill) {
        free(first); free(rows); free(fill);
        return -1;
    }
    for (int64_t v = 0; v < V; ++v)
        first[task_id[v] + 1] += 1;
    for (int64_t t = 0; t < T; ++t)
        first[t + 1] += first[t];
    for (int64_t v = 0; v < V; ++v) {
        int64_t t = task_id[v];
        rows[first[t] + fill[t]] = v;
        fill[t] += 1;
    }
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int32_t b = q_batch_idx[q];
        int64_t t = q_task[q];
        int64_t n = (b >= 0 && b < B && t >= 0 && t < T) ? first[t + 1] - first[t] : 0;
        case1_one(n ? rows + first[t] : rows, n, B, acc_bp, lat_us, cost, queue_us, state, load_us,
                  q_slo_us[q], q_min_acc_bp[q], b, &out_variant[q], &out_tier[q], &out_closest[q]);
    }
    free(first); free(rows); free(fill);
    return 0;
}

/* State report: state[row[i]] = value[i], in array order; entries with a row outside 0..V-1 or
 * a code outside 0..3 are skipped. */
void oracle_update_state(int64_t V, int32_t *state, int64_t n,
                         const int32_t *variant_idx, const int32_t *new_state)
{
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = variant_idx[i];
        if (v < 0 || v >= V || new_state[i] < 0 || new_state[i] > 3)
            continue;
        state[v] = new_state[i];
    }
}

/*
 * Worker selection (Section 4.1, Case I: the output of the policy is the variant AND the worker
 * that serves the query; Section 6.4 counts it as the second decision on the critical path).
 *
 *   The selected variant is Active   -> the query goes to the least-loaded worker that runs an
 *                                       instance of the variant;
 *   the selected variant is Inactive -> the query goes to the worker with the lowest utilisation
 *                                       among the workers that have the variant's target hardware;
 *   no variant                       -> no worker (-1).
 *
 * A running instance is a {variant, worker} pair (Section 5) with a load figure of its own.
 * Readings where the text is silent: "least loaded" compares the instances' load figures and, among
 * equal ones, takes the lower worker number; equal utilisations likewise go to the lower worker
 * number; an Active variant without any instance, or an Inactive one whose hardware no worker
 * has, gets worker -1 while the variant and tier stand; reports of utilisation or instance load
 * are applied in array order and skip entries with an index outside the table or a negative
 * value.
 */
static int32_t least_loaded_worker(int64_t n_inst, const int32_t *inst_variant,
                                   const int32_t *inst_worker, const int32_t *inst_load,
                                   const int64_t *list, int64_t n_list, int32_t variant)
{
    /* list == NULL: look at every instance; else only at the n_list instances listed */
    int64_t best = -1;
    int64_t count = list ? n_list : n_inst;
    for (int64_t j = 0; j < count; ++j) {
        int64_t i = list ? list[j] : j;
        if (inst_variant[i] != variant)
            continue;
        if (best < 0 || inst_load[i] < inst_load[best] ||
            (inst_load[i] == inst_load[best] && inst_worker[i] < inst_worker[best]))
            best = i;
    }
    return best >= 0 ? inst_worker[best] : -1;
}

static int32_t least_utilised_worker(int64_t W, const int32_t *worker_hw,
                                     const int32_t *worker_util, int32_t hw)
{
    int64_t best = -1;
    for (int64_t w = 0; w < W; ++w) {
        if (worker_hw[w] != hw)
            continue;
        if (best < 0 || worker_util[w] < worker_util[best])
            best = w;   /* equal utilisation: the earlier (lower) worker stays */
    }
    return (int32_t)best;
}

static int workers_args_ok(int64_t V, int64_t W, int64_t n_inst, const int32_t *inst_variant,
                           const int32_t *inst_worker)
{
    if (W < 0 || n_inst < 0)
        return 0;
    for (int64_t i = 0; i < n_inst; ++i)
        if (inst_variant[i] < 0 || inst_variant[i] >= V || inst_worker[i] < 0 || inst_worker[i] >= W)
            return 0;
    return 1;
}

/* Literal form: state-aware selection by the literal routine, then every instance / every worker
 * is looked at for every query. */
int oracle_select_workers_literal(int64_t V, int32_t B,
                                  const int32_t *task_id, const int32_t *acc_bp,
                                  const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                                  const int32_t *state, const int32_t *load_us,
                                  const int32_t *variant_hw,
                                  int64_t W, const int32_t *worker_hw, const int32_t *worker_util,
                                  int64_t n_inst, const int32_t *inst_variant,
                                  const int32_t *inst_worker, const int32_t *inst_load,
                                  int64_t N,
                                  const int32_t *q_task, const int32_t *q_slo_us,
                                  const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                                  int32_t *out_variant, int32_t *out_tier, int32_t *out_worker)
{
    if (!workers_args_ok(V, W, n_inst, inst_variant, inst_worker))
        return -1;
    int rc = oracle_select_tiered_literal(V, B, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                                          N, q_task, q_slo_us, q_min_acc_bp, q_batch_idx,
                                          out_variant, out_tier);
    if (rc != 0)
        return rc;
    for (int64_t q = 0; q < N; ++q) {
        if (out_tier[q] == 1)
            out_worker[q] = least_loaded_worker(n_inst, inst_variant, inst_worker, inst_load,
                                                NULL, 0, out_variant[q]);
        else if (out_tier[q] == 2)
            out_worker[q] = least_utilised_worker(W, worker_hw, worker_util,
                                                  variant_hw[out_variant[q]]);
        else
            out_worker[q] = -1;
    }
    return 0;
}

/* Grouped form: the instances are listed per variant once (as the rows are per task); each query
 * still walks the whole list of its variant, or all workers.  Queries on several host threads. */
int oracle_select_workers(int64_t V, int32_t B,
                          const int32_t *task_id, const int32_t *acc_bp,
                          const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                          const int32_t *state, const int32_t *load_us,
                          const int32_t *variant_hw,
                          int64_t W, const int32_t *worker_hw, const int32_t *worker_util,
                          int64_t n_inst, const int32_t *inst_variant,
                          const int32_t *inst_worker, const int32_t *inst_load,
                          int64_t N,
                          const int32_t *q_task, const int32_t *q_slo_us,
                          const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                          int32_t *out_variant, int32_t *out_tier, int32_t *out_worker)
{
    if (!workers_args_ok(V, W, n_inst, inst_variant, inst_worker))
        return -1;
    int rc = oracle_select_tiered(V, B, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                                  N, q_task, q_slo_us, q_min_acc_bp, q_batch_idx,
                                  out_variant, out_tier);
    if (rc != 0)
        return rc;
    int64_t *first = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *list = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_inst > 0 ? n_inst : 1));
    if (!first || !fill || !list) {
        free(first); free(fill); free(list);
        return -1;
    }
    for (int64_t i = 0; i < n_inst; ++i)
        first[inst_variant[i] + 1] += 1;
    for (int64_t v = 0; v < V; ++v)
        first[v + 1] += first[v];
    for (int64_t i = 0; i < n_inst; ++i) {
        int64_t v = inst_variant[i];
        list[first[v] + fill[v]] = i;
        fill[v] += 1;
    }
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int32_t v = out_variant[q];
        if (out_tier[q] == 1)
            out_worker[q] = least_loaded_worker(n_inst, inst_variant, inst_worker, inst_load,
                                                list + first[v], first[v + 1] - first[v], v);
        else if (out_tier[q] == 2)
            out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, variant_hw[v]);
        else
            out_worker[q] = -1;
    }
    free(first); free(fill); free(list);
    return 0;
}

/* Utilisation report: worker_util[idx[i]] = value[i], array order, invalid entries skipped. */
void oracle_update_worker_util(int64_t W, int32_t *worker_util, int64_t n,
                               const int32_t *worker_idx, const int32_t *new_util)
{
    for (int64_t i = 0; i < n; ++i) {
        int64_t w = worker_idx[i];
        if (w < 0 || w >= W || new_util[i] < 0)
            continue;
        worker_util[w] = new_util[i];
    }
}

/* Instance load report: inst_load[idx[i]] = value[i], array order, invalid entries skipped. */
void oracle_update_instance_load(int64_t n_inst, int32_t *inst_load, int64_t n,
                                 const int32_t *inst_idx, const int32_t *new_load)
{
    for (int64_t i = 0; i < n; ++i) {
        int64_t j = inst_idx[i];
        if (j < 0 || j >= n_inst || new_load[i] < 0)
            continue;
        inst_load[j] = new_load[i];
    }
}

/*
 * State per running instance (Section 4, "State machine for the lifecycle of model-variants": the
 * state is tracked per variant INSTANCE by the monitoring daemon of the worker that runs it;
 * Section 5 encodes an instance as a {variant, worker} pair).  A loaded instance is Active,
 * Overloaded or Interfered; a variant that runs nowhere is Inactive.  Case I (Section 4.1) then
 * reads:
 *
 *   a variant is looked at in the first step when at least one of its instances is Active, and the
 *   query goes to the least-loaded worker among those that run an ACTIVE instance of it (an
 *   Overloaded or Interfered instance is avoided even when another instance of the same variant
 *   serves);
 *   a variant without any instance is looked at in the second step, as before;
 *   a variant whose instances are all Overloaded or Interfered is not selected at all.
 *
 * Readings where the text is silent: the state of a variant with instances but no Active one is
 * reported as Overloaded when any instance is Overloaded, else Interfered (nothing depends on
 * which); instance state reports are applied in array order and skip entries whose index is
 * outside the table or whose code is not Active, Overloaded or Interfered (an instance cannot be
 * Inactive: it is loaded).
 */
int oracle_derive_states(int64_t V, int64_t n_inst, const int32_t *inst_variant,
                         const int32_t *inst_state, int32_t *out_state)
{
    for (int64_t i = 0; i < n_inst; ++i)
        if (inst_variant[i] < 0 || inst_variant[i] >= V)
            return -1;
    int64_t *running = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *active = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *overloaded = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    if (!running || !active || !overloaded) {
        free(running); free(active); free(overloaded);
        return -1;
    }
    for (int64_t i = 0; i < n_inst; ++i) {
        int64_t v = inst_variant[i];
        running[v] += 1;
        active[v] += inst_state[i] == STATE_ACTIVE;
        overloaded[v] += inst_state[i] == STATE_OVERLOADED;
    }
    for (int64_t v = 0; v < V; ++v) {
        if (running[v] == 0)
            out_state[v] = STATE_INACTIVE;
        else if (active[v] > 0)
            out_state[v] = STATE_ACTIVE;
        else
            out_state[v] = overloaded[v] > 0 ? STATE_OVERLOADED : STATE_INTERFERED;
    }
    free(running); free(active); free(overloaded);
    return 0;
}

/* Least-loaded worker among those that run an Active instance of the variant; equal loads go to
 * the lower worker number; -1 when there is none.  list == NULL: every instance is looked at;
 * else only the n_list instances listed. */
static int32_t least_loaded_active_worker(int64_t n_inst, const int32_t *inst_variant,
                                          const int32_t *inst_worker, const int32_t *inst_load,
                                          const int32_t *inst_state,
                                          const int64_t *list, int64_t n_list, int32_t variant)
{
    int64_t best = -1;
    int64_t count = list ? n_list : n_inst;
    for (int64_t j = 0; j < count; ++j) {
        int64_t i = list ? list[j] : j;
        if (inst_variant[i] != variant || inst_state[i] != STATE_ACTIVE)
            continue;
        if (best < 0 || inst_load[i] < inst_load[best] ||
            (inst_load[i] == inst_load[best] && inst_worker[i] < inst_worker[best]))
            best = i;
    }
    return best >= 0 ? inst_worker[best] : -1;
}

/* Case I with the state kept per instance: (variant, tier, worker) per query.  literal != 0: every
 * query walks all V rows and all instances; else the rows are listed per task and the instances
 * per variant once, and each query walks the lists of its own (queries on several host threads). */
int oracle_select_instances(int64_t V, int32_t B,
                            const int32_t *task_id, const int32_t *acc_bp,
                            const int32_t *lat_us, const int32_t *cost, const int32_t *queue_us,
                            const int32_t *load_us, const int32_t *variant_hw,
                            int64_t W, const int32_t *worker_hw, const int32_t *worker_util,
                            int64_t n_inst, const int32_t *inst_variant,
                            const int32_t *inst_worker, const int32_t *inst_load,
                            const int32_t *inst_state, int32_t literal,
                            int64_t N,
                            const int32_t *q_task, const int32_t *q_slo_us,
                            const int32_t *q_min_acc_bp, const int32_t *q_batch_idx,
                            int32_t *out_variant, int32_t *out_tier, int32_t *out_worker)
{
    if (!workers_args_ok(V, W, n_inst, inst_variant, inst_worker))
        return -1;
    for (int64_t i = 0; i < n_inst; ++i)
        if (inst_state[i] != STATE_ACTIVE && inst_state[i] != STATE_OVERLOADED && inst_state[i] != STATE_INTERFERED)
            return -1;
    int32_t *state = (int32_t *)malloc(sizeof(int32_t) * (size_t)(V > 0 ? V : 1));
    int64_t *first = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)calloc((size_t)V + 1, sizeof(int64_t));
    int64_t *list = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_inst > 0 ? n_inst : 1));
    int rc = (state && first && fill && list) ? 0 : -1;
    if (rc == 0)
        rc = oracle_derive_states(V, n_inst, inst_variant, inst_state, state);
    if (rc == 0)
        rc = literal ? oracle_select_tiered_literal(V, B, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                                                    N, q_task, q_slo_us, q_min_acc_bp, q_batch_idx, out_variant, out_tier)
                     : oracle_select_tiered(V, B, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                                            N, q_task, q_slo_us, q_min_acc_bp, q_batch_idx, out_variant, out_tier);
    if (rc != 0) {
        free(state); free(first); free(fill); free(list);
        return rc;
    }
    for (int64_t i = 0; i < n_inst; ++i)
        first[inst_variant[i] + 1] += 1;
    for (int64_t v = 0; v < V; ++v)
        first[v + 1] += first[v];
    for (int64_t i = 0; i < n_inst; ++i) {
        int64_t v = inst_variant[i];
        list[first[v] + fill[v]] = i;
        fill[v] += 1;
    }
#pragma omp parallel for schedule(dynamic, 4096)
    for (int64_t q = 0; q < N; ++q) {
        int32_t v = out_variant[q];
        if (out_tier[q] == 1)
            out_worker[q] = literal
                ? least_loaded_active_worker(n_inst, inst_variant, inst_worker, inst_load, inst_state, NULL, 0, v)
                : least_loaded_active_worker(n_inst, inst_variant, inst_worker, inst_load, inst_state,
                                             list + first[v], first[v + 1] - first[v], v);
        else if (out_tier[q] == 2)
            out_worker[q] = least_utilised_worker(W, worker_hw, worker_util, variant_hw[v]);
        else
            out_worker[q] = -1;
    }
    free(state); free(first); free(fill); free(list);
    return 0;
}

/* Instance state report: inst_state[idx[i]] = value[i], array order, invalid entries skipped. */
void oracle_update_instance_state(int64_t n_inst, int32_t *inst_state, int64_t n,
                                  const int32_t *inst_idx, const int32_t *new_state)
{
    for (int64_t i = 0; i < n; ++i) {
        int64_t j = inst_idx[i];
        if (j < 0 || j >= n_inst)
            continue;
        if (new_state[i] != STATE_ACTIVE && new_state[i] != STATE_OVERLOADED && new_state[i] != STATE_INTERFERED)
            continue;
        inst_state[j] = new_state[i];
    }
}

/*
 * Scaling decision on a change in query load (Section 4.2.2, "scaling up"; cost function and
 * constraints of the integer program of Section 4.2.1; instance counts and costs as in the
 * worked example of Section 2.2, Tables 2 and 3).
 *
 * A request names a running variant cur with n_cur instances, the incoming load L (queries per
 * second), the application's latency objective S and a batch index b.  With Q the saturation
 * throughput, C the hardware cost per second, T_load the loading latency of a variant and
 * T_inf = lat_us[.][b] its inference latency:
 *
 *   no action          when Q[cur] * n_cur already covers the load with the required headroom
 *                      (constraint 1; headroom = slack_pct percent of the load, the
 *                      slack-threshold of Section 5 is 1.05 = 105 percent);
 *   replicate          load d = inst(cur) - n_cur more instances of cur, allowed when
 *                      T_inf[cur] <= S (constraint 2 binds every newly loaded instance);
 *   upgrade            switch to a variant u of the same model architecture with T_inf[u] <= S
 *                      and Q[u] > Q[cur]: load inst(u) instances of u, unload the n_cur of cur;
 *   where inst(v) = ceil(L * slack_pct / (100 * Q[v])) instances of v alone carry the load.
 *
 * The options are compared by the integer program's objective, the sum over the touched variants
 * of  C * (delta + lambda * T_load * max(delta, 0)):
 *     replicate:  C[cur] * d * (1 + lambda * T_load[cur])
 *     upgrade:    C[u] * inst(u) * (1 + lambda * T_load[u])  -  C[cur] * n_cur
 * and the cheapest is taken.  Everything is an integer: lambda is per second and T_load in
 * microseconds, so all costs are carried times 1,000,000 and compared exactly in 128 bits.
 *
 * Readings where the text is silent: the cheapest upgrade wins ties by the lower row; replication
 * wins a tie against the cheapest upgrade (no switch without a gain); a request whose running
 * variant or batch index is outside the table, or with n_cur outside 0..1,000,000 or a load
 * outside 0..1,000,000,000 queries per second, gets no action (the limits keep every instance
 * count inside 32 bits; likewise lambda <= 1000 per second, slack_pct <= 200 and C <= 2^20);
 * when scaling is needed and neither option is allowed the action code is 3 (the worker has to
 * turn to the controller, step (d) of Section 4.2.2).  Resource limits of the worker
 * (constraint 3) are not part of this routine; scaling down is oracle_scale_down.
 *
 * Outputs per request: action (0 none, 1 replicate, 2 upgrade, 3 needed but impossible), the
 * variant to load (-1 for actions 0 and 3) and the number of its instances to load.
 */
typedef __int128 wide_t;

int oracle_scale(int64_t V, int32_t B,
                 const int32_t *arch_id, const int32_t *sat_qps, const int32_t *hw_cost,
                 const int32_t *load_us, const int32_t *lat_us,
                 int32_t lambda_per_s, int32_t slack_pct,
                 int64_t R,
                 const int32_t *r_variant, const int32_t *r_instances, const int32_t *r_load_qps,
                 const int32_t *r_slo_us, const int32_t *r_batch_idx,
                 int32_t *out_action, int32_t *out_variant, int32_t *out_instances)
{
    if (V < 0 || B <= 0 || R < 0 || lambda_per_s < 0 || lambda_per_s > 1000 || slack_pct < 0 ||
        slack_pct > 200)
        return -1;
    for (int64_t v = 0; v < V; ++v)
        if (sat_qps[v] < 1 || hw_cost[v] < 0 || hw_cost[v] > 1048576 || load_us[v] < 0)
            return -1;
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t r = 0; r < R; ++r) {
        int64_t cur = r_variant[r];
        int32_t b = r_batch_idx[r];
        out_action[r] = 0;
        out_variant[r] = -1;
        out_instances[r] = 0;
        if (cur < 0 || cur >= V || b < 0 || b >= B || r_instances[r] < 0 || r_load_qps[r] < 0 ||
            r_instances[r] > 1000000 || r_load_qps[r] > 1000000000)
            continue;
        int64_t n_cur = r_instances[r];
        int64_t need = (int64_t)r_load_qps[r] * (int64_t)slack_pct;        /* hundredths of a query per second */
        if ((int64_t)sat_qps[cur] * n_cur * 100 >= need)
            continue;                                                       /* constraint 1 holds already */
        int64_t slo = r_slo_us[r];
        int have = 0;
        int64_t best_v = -1, best_n = 0;
        wide_t best_cost = 0;
        if ((int64_t)lat_us[cur * B + b] <= slo) {                          /* replicate */
            int64_t per = 100 * (int64_t)sat_qps[cur];
            int64_t inst = (need + per - 1) / per;
            best_n = inst - n_cur;
            best_v = cur;
            best_cost = (wide_t)hw_cost[cur] * best_n *
                        ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[cur]);
            have = 1;
        }
        wide_t saved = (wide_t)hw_cost[cur] * n_cur * 1000000;              /* unloading cur */
        for (int64_t u = 0; u < V; ++u) {                                   /* upgrade */
            if (u == cur || arch_id[u] != arch_id[cur])
                continue;
            if ((int64_t)lat_us[u * B + b] > slo || sat_qps[u] <= sat_qps[cur])
                continue;
            int64_t per = 100 * (int64_t)sat_qps[u];
            int64_t inst = (need + per - 1) / per;
            wide_t cost = (wide_t)hw_cost[u] * inst *
                          ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - saved;
            if (!have || cost < best_cost) {        /* rows ascend: an equal cost keeps the earlier choice */
                best_cost = cost;
                best_v = u;
                best_n = inst;
                have = 1;
            }
        }
        if (!have) {
            out_action[r] = 3;
            continue;
        }
        out_action[r] = best_v == cur ? 1 : 2;
        out_variant[r] = (int32_t)best_v;
        out_instances[r] = (int32_t)best_n;
    }
    return 0;
}

/*
 * Scaling down (Section 4.2.2, "Scaling down algorithm").
 *
 * At regular intervals the selection policy is asked whether the incoming load L of a running
 * variant cur with n_cur instances can be carried for less: by removing an instance of cur, or by
 * downgrading to a cheaper variant.  Per request (cur, n_cur, L, S, b):
 *   remove             unload one instance of cur, allowed when at least one stays and the rest
 *                      still carries the load with the required headroom,
 *                      Q[cur] * (n_cur - 1) * 100 >= L * slack_pct  (constraint 1);
 *   downgrade          switch to a variant u of the same model architecture with a lower hardware
 *                      cost, C[u] < C[cur], and T_inf[u] <= S (constraint 2 binds every newly loaded
 *                      instance): load inst(u) = max(1, ceil(L * slack_pct / (100 * Q[u])))
 *                      instances of u, which carry the load by construction, unload the n_cur of cur;
 *   keep               otherwise.
 * The options are compared by the integer program's objective, as in scaling up:
 *     keep:       0
 *     remove:     - C[cur]                                       (delta = -1, nothing is loaded)
 *     downgrade:  C[u] * inst(u) * (1 + lambda * T_load[u])  -  C[cur] * n_cur
 * and the lowest is taken; only an option that lowers the objective is acted on.
 *
 * Readings where the text is silent: one instance is removed per decision; the last instance is
 * never removed here (unloading a variant altogether is the state machine's business, Section 4);
 * a downgrade keeps at least one instance serving even when no load arrives; ties go to keeping,
 * then to removing, then to the lower row among downgrades (no switch without a gain); invalid
 * requests as in scaling up.  The wait of T_v = T_load[cur] before the action is executed is the
 * caller's: the decision does not depend on it.
 *
 * Outputs per request: action (0 keep, 1 remove, 2 downgrade), the variant concerned (cur for 1,
 * u for 2, -1 for 0) and the instances of it to unload (1, action 1) or to load (inst(u), action 2).
 */
int oracle_scale_down(int64_t V, int32_t B,
                      const int32_t *arch_id, const int32_t *sat_qps, const int32_t *hw_cost,
                      const int32_t *load_us, const int32_t *lat_us,
                      int32_t lambda_per_s, int32_t slack_pct,
                      int64_t R,
                      const int32_t *r_variant, const int32_t *r_instances, const int32_t *r_load_qps,
                      const int32_t *r_slo_us, const int32_t *r_batch_idx,
                      int32_t *out_action, int32_t *out_variant, int32_t *out_instances)
{
    if (V < 0 || B <= 0 || R < 0 || lambda_per_s < 0 || lambda_per_s > 1000 || slack_pct < 0 ||
        slack_pct > 200)
        return -1;
    for (int64_t v = 0; v < V; ++v)
        if (sat_qps[v] < 1 || hw_cost[v] < 0 || hw_cost[v] > 1048576 || load_us[v] < 0)
            return -1;
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t r = 0; r < R; ++r) {
        int64_t cur = r_variant[r];
        int32_t b = r_batch_idx[r];
        out_action[r] = 0;
        out_variant[r] = -1;
        out_instances[r] = 0;
        if (cur < 0 || cur >= V || b < 0 || b >= B || r_instances[r] < 0 || r_load_qps[r] < 0 ||
            r_instances[r] > 1000000 || r_load_qps[r] > 1000000000)
            continue;
        int64_t n_cur = r_instances[r];
        int64_t need = (int64_t)r_load_qps[r] * (int64_t)slack_pct;        /* hundredths of a query per second */
        int64_t slo = r_slo_us[r];
        wide_t lowest = 0;                                                  /* keeping everything */
        if (n_cur >= 2 && (int64_t)sat_qps[cur] * (n_cur - 1) * 100 >= need) {   /* remove one */
            wide_t objective = -(wide_t)hw_cost[cur] * 1000000;
            if (objective < lowest) {
                lowest = objective;
                out_action[r] = 1;
                out_variant[r] = (int32_t)cur;
                out_instances[r] = 1;
            }
        }
        wide_t unloaded = (wide_t)hw_cost[cur] * n_cur * 1000000;          /* all of cur */
        for (int64_t u = 0; u < V; ++u) {                                   /* downgrade */
            if (u == cur || arch_id[u] != arch_id[cur])
                continue;
            if ((int64_t)lat_us[u * B + b] > slo || hw_cost[u] >= hw_cost[cur])
                continue;
            int64_t per = 100 * (int64_t)sat_qps[u];
            int64_t inst = (need + per - 1) / per;
            if (inst < 1)
                inst = 1;
            wide_t objective = (wide_t)hw_cost[u] * inst *
                               ((wide_t)1000000 + (wide_t)lambda_per_s * load_us[u]) - unloaded;
            if (objective < lowest) {               /* rows ascend: an equal objective keeps the earlier choice */
                lowest = objective;
                out_action[r] = 2;
                out_variant[r] = (int32_t)u;
                out_instances[r] = (int32_t)inst;
            }
        }
    }
    return 0;
}

/* Host threads the grouped form uses. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Host threads the grouped forms are to use from now on (n < 1: leave as is); returns what they use then. */
int oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#endif
    return oracle_num_threads();
}
