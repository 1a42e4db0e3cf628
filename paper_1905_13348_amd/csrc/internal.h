// Internal declarations shared by the host runtime and the kernel files of libinfaas_sel.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace infaas {

constexpr int kQueriesPerTile = 512;     // queries that share one staged slice in the scan
constexpr uint32_t kNoRank = 0xFFFFFFFFu; // "no feasible variant" in rank space
constexpr int kLdsHistMaxSlices = 8192;   // per-workgroup LDS histogram up to this many slices

// Variant store as the kernels see it.  "slot" = position in the task-sorted, 4-padded
// layout; a task's segment starts at seg_off[t] (multiple of 4) and has seg_len[t] rows.
struct TableView {
    int32_t T, B, S, V, Vp;
    int32_t lds_limit;          // variants per staged chunk; segments above it take the wide path
    const int32_t *acc;         // [Vp]
    int32_t *queue;             // [Vp]
    const int32_t *orig;        // [Vp] caller row of each slot
    const int32_t *lat;         // [B][Vp]
    const uint32_t *rank;       // [B][Vp] position of the slot in its slice's (cost, lat, row) order
    const uint32_t *perm;       // [B][Vp] inverse: perm[b][seg+r] = slot-in-segment of rank r
    const int32_t *seg_off;     // [T+1]
    const int32_t *seg_len;     // [T]
    const int32_t *slot_of;     // [V] caller row -> slot
    // The same slices once more, stored in rank order: entry seg_off[t] + r of column b is the
    // variant of rank r in slice (t, b).  tot_r = lat_r + queue is kept current by load updates.
    int32_t *acc_r;             // [B][Vp]
    uint32_t *tot_r;            // [B][Vp]
    const int32_t *lat_r;       // [B][Vp]
    const int32_t *orig_r;      // [B][Vp] caller row
    const int32_t *gpos;        // [B][Vp] slot -> its entry in the rank-ordered column b
    int32_t acc_base;           // smallest accuracy in the table; index keys are acc - acc_base + 1
    // State-aware selection: a table serves one state (Active or Inactive).  Variants in another
    // state are masked in the rank-ordered columns (accuracy = acc_base, latency-plus-queue =
    // 0xFFFFFFFF): nothing selects them and every entry ranked before them dominates them.
    int32_t *state;             // [Vp] state of each slot, or null when the table is not state-aware
    int32_t want_state;         // the state this table serves
    // Six counters of the latest build of the table's index (kCtlMaxK0 .. kCtlMaxK, kCtlPool, kCtlSteps) and
    // where the first kernel of every selection copies them for the host to see (pinned host memory); null: nowhere.
    const uint32_t *stat_src;
    uint32_t *stat_dst;
};

// ---------------------------------------------------------------- staircase index
//
// For one (task, batch) slice, walk the variants in rank order and keep a variant only if no
// earlier (cheaper) one has at least its accuracy and at most its latency-plus-queue: a query
// that the later one satisfies is also satisfied by the earlier one, which wins.  The kept
// variants ("steps") are the only possible answers, and the answer to (min_acc, slo) is the
// first step with acc >= min_acc and tot <= slo.
//
// Steps are stored in groups of at most 31 ("bodies"; a slice has up to two).  Within a body
// the first fitting step is
//     ctz( A[#steps with acc >= min_acc] & S[#steps with tot <= slo] )
// where A[p] / S[p] are 32-bit sets (over the body's step numbers) of its p most accurate /
// p fastest steps.  Both counts come from a 5-probe binary search over a sorted copy of the
// keys.  Only when the first body has no fitting step is the second one consulted.
//
// Body with K steps: Re keys per sorted array, Re = K + 1 rounded up to even (the keys of the
// steps, then one or two sentinels).  Byte offsets from the body start, which is 4-byte aligned:
//   0            acc16 : u16[Re]  acc - acc_base + 1, descending; then 0 (sentinels)
//   2 Re         totk  : u32[Re]  tot, ascending; then 0xFFFFFFFF (sentinels)
//   6 Re         A     : u32[Re]  A[0] = 0, A[p] for p = 1..K
//   10 Re        S     : u32[Re]  S[0] = 0, S[p] for p = 1..K
// (when Re = K + 2 the last entry of A and of S repeats the full set, so that every entry is valid)
// A slice's block in the pool is  [rows][first body][second body]:  rows holds the low 16 bits
// of the caller rows of the first r = min(K, hot_rows) steps of the first body, in REVERSE order
// and padded in front to 4 bytes, so that those of step i are at (first body start) - 2 - 2 i.
// The bits above (row_hi_bits per step, as many as the table's row numbers need) sit in the
// header, step i at bit i * row_hi_bits of a 14-bit field, which limits hot_rows to
// 14 / row_hi_bits.  Deeper steps are translated through step_row in global memory.
// Headers hold "body start - 4" (called the body address below), so that accuracy key j (1-based)
// is at address + 2 + 2j, latency key j at address + 2 Re + 4j and the row of step i at
// address + 2 - 2i.
constexpr int kBodySteps = 31;               // steps per body
constexpr int kIndexCap = 2 * kBodySteps;    // steps kept per slice; more => slice marked truncated
constexpr uint32_t kHdrK0Shift = 16;         // header word y: bits 0-13 high row bits (global) / bits 0-15 first step_row entry (LDS copy),
constexpr uint32_t kHdrK1Shift = 22;         //   bits 16-21 Re of body 0, bits 22-27 Re of body 1 (0 = none)
constexpr uint32_t kHdrTrunc = 1u << 28;     // steps beyond the capacity exist: a miss in both bodies proves nothing
constexpr uint32_t kHdrPark = 1u << 29;      // no usable body: every query of the slice takes the slow path
constexpr uint32_t kLdsAddrBits = 18;        // LDS copy of a header: x = body address | high row bits << 18
constexpr uint32_t kRowHiField = 32 - kLdsAddrBits;   // bits for the high row bits of the first steps
constexpr uint32_t kHdrDeep = 1u << 31;      // a miss in the first body is not final (second body, truncation or
                                             // no usable body); the sign bit, so that one compare tests it
constexpr uint32_t kLdsHdrBytes = 8;         // per slice in the lookup kernel's LDS: {body address, y | first step}
constexpr uint32_t kLdsCtrlBytes = 48;       // control words at the start of the lookup kernel's LDS: 2 next unit, 3 records
                                             // in the open list, 4..8 the statistics below
constexpr int kLookupStats = 5;              // per launch and workgroup: queries parked; of those, answered by a second body,
                                             // by a first body read from global memory, sent through the rank-ordered
                                             // scan, and left without an answer

// LDS bytes of the S + 1 slice headers, padded so that the bodies behind them are 16-byte aligned
__host__ __device__ inline uint32_t lds_header_bytes(int32_t S) { return (((uint32_t)S + 1u) * kLdsHdrBytes + 15u) & ~15u; }
__host__ __device__ inline uint32_t body_re(uint32_t steps) { return (steps + 2u) & ~1u; }   // Re of a body with `steps` steps
__host__ __device__ inline uint32_t body_bytes(uint32_t re) { return 14u * re; }

struct IndexView {
    uint4 *hdr;          // [S + 1] {body address (pool offset - 4), y (see kHdr*), first entry in step_row, end of bodies};
                         //         entry S is the header of an empty slice, used for queries outside the table
    uint8_t *pool;       // bodies; an empty dummy body sits at offset 4 (its address is 0)
    uint32_t pool_bytes;
    int32_t *step_row;   // caller row of every step; entry 0 is unused
    int32_t *step_worker;// worker that serves the row of every step (worker selection), else null; entry 0 is -1
    uint16_t *hot_worker;// [S][hot_rows] the same for the first hot_rows steps of every slice, 0xFFFF for -1, for
                         // the lookup kernel's LDS; null when there are no hot rows or workers above 65534
    uint32_t step_cap;
    uint32_t hot_rows;   // rows kept in front of the first body of every slice (fills the LDS left over)
    uint32_t row_hi_bits;// bits of a row number above its low 16
    uint32_t *ctrl;      // [kCtlWords] counters of the build, see kCtl*
    unsigned long long *slice_room;   // [S] what slice s needs, published by the build that places the slices in the
                         // order of their numbers: steps << 32 | build number (12 bits) << 20 | bytes
    // Groups.  When the bodies of all slices do not fit one compute unit's LDS, the tasks are dealt, in
    // order, to num_groups groups whose bodies do: group g owns the tasks [group_task0[g],
    // group_task0[g + 1]), the bytes [g * region_bytes, (g + 1) * region_bytes) of the pool (every region
    // starts with a copy of the empty dummy body) and the entries [g * group_step_cap, ...) of step_row;
    // a slice that finds its group's region full is stored behind the regions.  num_groups == 1: one
    // region, the whole pool.
    uint32_t num_groups, region_bytes, group_step_cap;
    const uint16_t *task_group;   // [T] group of every task; null when num_groups == 1
    const int32_t *group_task0;   // [num_groups + 1]
    uint32_t *gctrl;              // [2 num_groups] per group: bytes of its region and steps handed out
    uint32_t *stats;     // [workgroups of the lookup kernel][kLookupStats] what the most recent lookup launch did
};
// Counters of the index build.  Every slice takes its room with one 64-bit add on the pair
// (kCtlPool, kCtlSteps) and waits for the answer; the statistics live on a cache line of their
// own so that their updates, which nobody waits for, do not queue in front of those requests.
constexpr int kCtlPool = 0;       // bytes of the pool handed out (with groups: behind the regions)
constexpr int kCtlSteps = 1;      // entries of step_row handed out (entry 0 is unused)
constexpr int kCtlPool0 = 8;      // what the two counters above start from at every rebuild
constexpr int kCtlSteps0 = 9;
constexpr int kCtlEpoch = 10;     // number of the build (12 bits), so that what earlier builds left in slice_room is told apart
constexpr int kCtlMaxK0 = 32;     // most steps in a first body (sets the probe count of the lookup)
constexpr int kCtlTrunc = 33;     // slices with more steps than the index keeps
constexpr int kCtlNoBody = 34;    // slices without a body
constexpr int kCtlMaxK = 35;      // most steps in a slice
constexpr int kCtlWords = 64;
// Called by every thread of the first kernel of a selection.
__device__ __forceinline__ void publish_index_stats(const TableView &tv)
{
    if (tv.stat_dst && blockIdx.x == 0 && threadIdx.x < 6)   // words 4, 5: pool bytes and step_row entries handed out
        tv.stat_dst[threadIdx.x] = tv.stat_src[threadIdx.x < 4 ? kCtlMaxK0 + threadIdx.x : kCtlPool + (threadIdx.x - 4)];
}

constexpr uint32_t kDummyBodyBytes = 64;     // 4 unused bytes, the empty body (28 bytes), padding
constexpr uint32_t kEmptyHdrY = 2u << kHdrK0Shift;  // Re = 2 (sentinels only), no second body

// Scratch of the scan engine for one pass over up to `capacity` queries.
struct ScanScratch {
    int32_t *cnt;        // [S]   queries per slice
    int32_t *bucket_off; // [S+1] exclusive prefix of cnt
    int32_t *cursor;     // [S]   running insert position per slice
    int32_t *tile_off;   // [S+1] exclusive prefix of LDS-path tiles per slice
    int32_t *wide_off;   // [S+1] exclusive prefix of wide-path work items per slice
    int32_t *counters;   // [4]   work-queue heads: 0 = LDS tiles, 1 = wide items
    int4 *recs;          // [capacity] bucketed queries {slo, min_acc, query id, slice}
    uint32_t *best;      // [capacity] device-wide minima of the wide path (rank space)
};

struct QueryView {
    int32_t n;
    const int32_t *task, *slo, *min_acc, *bidx;
    int32_t *out;
    int32_t *closest;    // second result array of the closest-variant mode, else null
    int32_t *tier;       // tier array of the state-aware selection, else null
    // state-aware selection: the lists of queries the first tier leaves open, one per workgroup of
    // the lookup kernel (open_cap records of 16 bytes each), and the number of records in each
    int32_t *open, *open_count;
    int32_t open_cap;
    // complete Case I: beside every record of those lists, what the first tier suggests for the query and
    // how far that variant is from the requirements (16 bytes: row or -1, latency beyond the bound, accuracy
    // below the bound, requirements missed | the 33rd bits), so that the second tier need not look it up
    int32_t *open_side;
    // worker selection: third result array, and the worker of every caller row for the tier the
    // pass looks at (for answers that do not come from a step of the index)
    int32_t *worker;
    const int32_t *row_worker;
    int32_t pass;        // 0 selection, 1 with closest-variant suggestion, 2 / 3 first / second tier, 4 / 5 the same with
                         // workers, 6 / 7 the tiers of the complete Case I (suggestion where neither tier answers)
};

// A pair of events that a launcher attaches to its kernel's dispatch (the events then carry the
// kernel's own start and end time, without the gaps that separately recorded events include).
struct LaunchEvents {
    hipEvent_t start, stop;
};

// Launches `kernel`, with the events attached when ev is not null.
template <class... P, class... A>
inline hipError_t launch_kernel(const LaunchEvents *ev, void (*kernel)(P...), dim3 grid, dim3 block, size_t lds,
                                hipStream_t st, A... args)
{
    if (ev) hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, ev->start, ev->stop, 0u, static_cast<P>(args)...);
    else hipLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, static_cast<P>(args)...);
    return hipGetLastError();
}

// Kernel launchers (scan engine).  Each returns the hipError_t of its launch.
// index: the index that is rebuilt afterwards (its allocator counters are rewound), or null.
hipError_t launch_update_load(const TableView &tv, int32_t n, const int32_t *idx,
                              const int32_t *val, const IndexView *index, hipStream_t st, const LaunchEvents *ev = nullptr);
// State report: state of row idx[i] := val[i] (idx null: row i, all V rows), masks refreshed.
hipError_t launch_update_state(const TableView &tv, int32_t n, const int32_t *idx,
                               const int32_t *val, const IndexView *index, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_histogram(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_plan(const TableView &tv, const ScanScratch &sc, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_scatter(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                          bool init_best, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_scan_lds(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                           int32_t max_lds_segment, int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_scan_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_finish_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                              hipStream_t st, const LaunchEvents *ev = nullptr);
// q.closest from q.out: the selection where there is one, else the closest variant of the query's slice by an
// exhaustive scan (handles without the staircase index).
hipError_t launch_closest_scan(const TableView &tv, const QueryView &q, int num_cus, hipStream_t st,
                               const LaunchEvents *ev = nullptr);

// Kernel launchers (staircase index).
hipError_t launch_index_build(const TableView &tv, const IndexView &ix, hipStream_t st, const LaunchEvents *ev = nullptr);
// lds_bytes: dynamic LDS of the lookup kernel when the index is mirrored in LDS, 0 to read it
// from global memory.  park_mem: index_park_bytes() of device memory (16-byte aligned) for the
// queues of parked queries; its size does not depend on the number of queries.
hipError_t launch_index_select(const TableView &tv, const IndexView &ix, const QueryView &q,
                               int32_t *park_mem, uint32_t lds_bytes, int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);
int index_select_blocks(int num_cus);
int32_t index_open_cap(int32_t n, int num_cus);   // records per workgroup of QueryView::open for a pass over n queries
size_t index_park_bytes(int num_cus);

// Selection group by group, for an index laid out in groups (IndexView::num_groups > 1).
constexpr int kGroupTile = 16384;   // queries binned at a time
struct GroupScratch {
    uint2 *rec;          // [tiles * kGroupTile] records {latency bound, accuracy threshold (key space) | slice in its group << 16},
                         //   the records of a tile grouped by group
    uint16_t *perm;      // [tiles * kGroupTile] query -> where its record sits in its tile
    int32_t *res;        // [tiles * kGroupTile] answers, in record order
    uint32_t *desc;      // [tiles][groups + 1] the tile's run of every group: offset in the tile | length << 15
    uint32_t *gcount;    // [groups + 1] records per group (cleared again by the last kernel of a call)
    int32_t max_group_slices;   // slices of the largest group
    int32_t stat_blocks;        // workgroups IndexView::stats has room for
};
size_t group_bin_lds_bytes(int32_t T, int32_t G);
hipError_t launch_group_bin(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                            int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_group_lookup(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                               int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_group_finish(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                               int num_cus, hipStream_t st, const LaunchEvents *ev = nullptr);

// Worker selection (Section 4.1: the worker that serves the selected variant).
struct WorkerView {
    int32_t V, W, I, H;           // variants, workers, instances, hardware classes that have workers
    int32_t *util;                // [W] utilisation, caller's worker numbers
    const int32_t *cls_off;       // [H + 1] workers grouped by hardware class ...
    const int32_t *cls_worker;    // [W]     ... worker numbers, ascending inside a class
    const int32_t *var_cls;       // [V] class of the variant's target hardware, -1 when no worker has it
    const int32_t *inst_off;      // [V + 1] instances grouped by variant (caller row) ...
    const int32_t *inst_worker;   // [I]     ... their workers
    int32_t *inst_load;           // [I]     ... their loads
    int32_t *inst_state;          // [I]     ... their states (Active, Overloaded, Interfered), or null: all Active
    int32_t *derived;             // [V] with instance states: the state of every variant as its instances give it
    const int32_t *inst_pos;      // [I] caller's instance number -> position in the grouped arrays
    int32_t *best_cls;            // [H] least-utilised worker of every class
    int32_t *row_worker;          // [2 V] worker by caller row: for an Active answer, then for an Inactive one
};
// Utilisation and instance-load report (either part may be empty).
hipError_t launch_worker_report(const WorkerView &wv, int32_t n, const int32_t *worker_idx, const int32_t *util,
                                int32_t m, const int32_t *inst_idx, const int32_t *load, hipStream_t st,
                                const LaunchEvents *ev = nullptr);
// Instance state report: the state of instance inst_idx[i] = state[i]; entries outside the table or with a
// code that is not Active, Overloaded or Interfered are skipped.
hipError_t launch_instance_state_report(const WorkerView &wv, int32_t n, const int32_t *inst_idx, const int32_t *state,
                                        hipStream_t st, const LaunchEvents *ev = nullptr);
// wv.derived from wv.inst_state: Inactive without instances, Active with an Active one, else Overloaded if
// some instance is, else Interfered.
hipError_t launch_derive_states(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev = nullptr);
// best_cls, then row_worker, from the current utilisations and loads (in this order).
hipError_t launch_best_per_class(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev = nullptr);
hipError_t launch_worker_tables(const WorkerView &wv, hipStream_t st, const LaunchEvents *ev = nullptr);
// ix.step_worker[j] = row_worker[ix.step_row[j]] for every step of the index (row_worker: num_rows entries).
hipError_t launch_step_workers(const IndexView &ix, const int32_t *row_worker, int32_t num_rows, hipStream_t st,
                               const LaunchEvents *ev = nullptr);
// ix.hot_worker from ix.step_worker (num_slices = S of the table the index belongs to); no-op without hot_worker.
hipError_t launch_hot_workers(const IndexView &ix, int32_t num_slices, hipStream_t st, const LaunchEvents *ev = nullptr);

// Scaling decision on a change in load (Section 4.2.2).
// Everything a request reads sits in ONE 128-byte block per (batch size, caller row) -- 32 words:
//   0 saturation throughput Q of the row, 1 its hardware cost, 2-3 the cost of one loaded instance
//   C * (1,000,000 + lambda * T_load), 4 its inference latency at the batch size, 5 the number m of
//   candidates for an upgrade (those of its architecture's list with a higher throughput: a prefix
//   of the list), 6 where that list starts in `cand`, 7 | 28-31 the caller rows of
//   the first five candidates (the fifth in word 7), 8-27 those candidates, four words each.
// Candidates beyond the fifth are read from the shared list.
constexpr int kScaleBlockWords = 32;
constexpr int kScaleInBlock = 5;
struct ScaleCand {    // one candidate for an upgrade, as the shared lists hold it
    uint32_t qps;     // saturation throughput
    int32_t lat;      // inference latency at the list's batch size
    uint64_t unit;    // cost of one loaded instance
    int32_t row;      // caller row
    int32_t pad[3];
};
struct ScaleView {
    int32_t V, B;             // variants, batch sizes
    int32_t slack_pct;
    const uint32_t *blocks;   // [B][V][32]
    const ScaleCand *cand;    // per (batch size, architecture) the variants that can ever win an upgrade, by
                              // descending throughput
    // The same two for scaling down: the candidates of a row are those for a downgrade (the prefix with a
    // lower hardware cost of its architecture's list, which is sorted by ascending hardware cost).
    const uint32_t *blocks_down;
    const ScaleCand *cand_down;
};
// down: the scaling-down decision (keep, remove an instance, downgrade) instead of scaling up
hipError_t launch_scale(const ScaleView &sv, bool down, int64_t R, const int32_t *r_variant, const int32_t *r_instances,
                        const int32_t *r_load_qps, const int32_t *r_slo_us, const int32_t *r_batch_idx,
                        int32_t *out_action, int32_t *out_variant, int32_t *out_instances, int num_cus,
                        hipStream_t st, const LaunchEvents *ev = nullptr);

}  // namespace infaas
