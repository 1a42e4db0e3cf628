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
    // The same slices once more, stored in rank order: entry seg_off[t] + r of column b is the
    // variant of rank r in slice (t, b).  tot_r = lat_r + queue is kept current by load updates.
    const int32_t *acc_r;       // [B][Vp]
    uint32_t *tot_r;            // [B][Vp]
    const int32_t *lat_r;       // [B][Vp]
    const int32_t *orig_r;      // [B][Vp] caller row
    const int32_t *gpos;        // [B][Vp] slot -> its entry in the rank-ordered column b
};

// ---------------------------------------------------------------- staircase index
//
// For one (task, batch) slice, walk the variants in rank order and keep a variant only if no
// earlier (cheaper) one has at least its accuracy and at most its latency-plus-queue: a query
// that the later one satisfies is also satisfied by the earlier one, which wins.  The kept
// variants ("steps") are the only possible answers, and the answer to (min_acc, slo) is the
// first step with acc >= min_acc and tot <= slo.  With K <= 63 steps that is
//     ctz( A[#steps with acc >= min_acc] & S[#steps with tot <= slo] )
// where A[p] / S[p] are bit sets (over step numbers) of the p most accurate / p fastest steps.
// Both counts come from a binary search over a sorted copy of the keys.
//
// Body of one slice (byte offsets from the body start; every section 4-byte aligned):
//   acc16 : u16[K+1]  acc - base + 1, descending, then a 0 sentinel
//   totk  : u32[K+1]  tot, ascending, then a 0xFFFFFFFF sentinel
//   ra    : u8[K]     step number of the j-th most accurate step
//   rs    : u8[K]     step number of the j-th fastest step
//   ea    : (u32 x W)[K/2]  A[2], A[4], ...   (W = 2 when K > 32; odd counts add one bit via ra)
//   es    : (u32 x W)[K/2]  S[2], S[4], ...
constexpr int kIndexCap = 63;            // steps kept per slice; more => slice marked truncated
constexpr uint32_t kHdrWide = 1u << 8;   // 64-bit masks
constexpr uint32_t kHdrTrunc = 1u << 9;  // steps beyond the capacity exist: an empty mask proves nothing
constexpr uint32_t kHdrIndexed = 1u << 10;  // body and step table are valid
constexpr uint32_t kHdrPark = 1u << 11;  // no usable body: every query of the slice takes the slow path
constexpr uint32_t kHdrBytes = 32;       // two uint4 per slice, see IndexView::hdr
constexpr uint32_t kLdsCtrlBytes = 16;   // control words at the start of the lookup kernel's LDS
constexpr uint32_t kBodySlack = 8;       // bytes after every body that unconditional reads may touch
constexpr int kIndexTile = 4096;         // queries per workgroup step of the index lookup kernel

struct BodyLayout {
    uint32_t o_tot, o_ra, o_rs, o_ea, o_es, size;
    __host__ __device__ BodyLayout(uint32_t K, uint32_t wide)
    {
        const uint32_t k1 = K + 1, rk = (K + 3) & ~3u, e = (K >> 1) << (wide ? 3 : 2);
        o_tot = (2 * k1 + 3) & ~3u;
        o_ra = o_tot + 4 * k1;
        o_rs = o_ra + rk;
        o_ea = o_rs + rk;
        o_es = o_ea + e;
        size = o_es + e + kBodySlack;
    }
};

struct IndexView {
    uint4 *hdr;          // [2S] per slice: {acc keys - 2, tot keys - 4, ea - 1 entry, es - 1 entry} (byte offsets in pool),
                         //               {K + 1 | flags, acc base, first entry in step_row, body end}
    uint8_t *pool;       // bodies; a dummy K=1 body sits at offset 0
    uint32_t pool_bytes;
    int32_t *step_row;   // caller row of every step
    uint32_t step_cap;
    uint32_t *ctrl;      // [0] pool bump, [1] step bump, [2] max K, [3] truncated slices,
                         // [4] slices without body, [5] total steps
};
constexpr uint32_t kDummyBodyBytes = 64;

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
                              const int32_t *val, uint32_t *index_ctrl, hipStream_t st);
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

// Kernel launchers (staircase index).
hipError_t launch_index_build(const TableView &tv, const IndexView &ix, hipStream_t st);
// lds_bytes: dynamic LDS of the lookup kernel when the index is mirrored in LDS, 0 to read it
// from global memory.  defer_q holds at least n + blocks * kIndexTile entries.
hipError_t launch_index_select(const TableView &tv, const IndexView &ix, const QueryView &q,
                               int32_t *defer_q, uint32_t lds_bytes, int num_cus, hipStream_t st);
int index_select_blocks(int num_cus);

}  // namespace infaas
