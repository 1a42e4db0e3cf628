// Internal declarations shared by the host runtime and the kernel files of libinfaas_sel.
#pragma once

#include <hip/hip_runtime.h>
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
};

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
};

// Kernel launchers (scan engine).  Each returns the hipError_t of its launch.
hipError_t launch_update_load(const TableView &tv, int32_t n, const int32_t *idx,
                              const int32_t *val, uint32_t *dirty_tasks, hipStream_t st);
hipError_t launch_histogram(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            hipStream_t st);
hipError_t launch_plan(const TableView &tv, const ScanScratch &sc, hipStream_t st);
hipError_t launch_scatter(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                          bool init_best, hipStream_t st);
hipError_t launch_scan_lds(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                           int32_t max_lds_segment, int num_cus, hipStream_t st);
hipError_t launch_scan_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            int num_cus, hipStream_t st);
hipError_t launch_finish_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                              hipStream_t st);

}  // namespace infaas
