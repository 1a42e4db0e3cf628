// The selection (Section 4.1 of the INFaaS paper) for tables whose staircase index does not fit
// one compute unit's LDS.  The tasks are dealt to groups whose bodies do fit (IndexView, internal.h),
// and a large batch of queries is answered in three passes:
//
//   k_group_bin    : tile by tile (16,384 queries), every query becomes an 8-byte record {latency
//                    bound, accuracy threshold in key space | slice inside its group} and the
//                    records of a tile are written grouped by group ("runs"); a 16-bit
//                    permutation remembers where each query's record went
//   k_group_lookup : the workgroups are dealt to the groups in proportion to their records; a
//                    workgroup mirrors ITS group's bodies in LDS and answers that group's runs
//                    with the same two binary searches and set intersection as k_index_select,
//                    records in, answers out, both coalesced
//   k_group_finish : puts the answers back into query order; the few queries the first body of their
//                    slice could not decide are finished here from the index in global memory
//
// Per query this moves 48 bytes instead of the 20 a table that fits in LDS needs, all of it
// streamed; the alternative, ten dependent probes per query into an index that lives in L2, is
// bound by the rate at which a compute unit can issue scattered loads and was 4 times slower.
#include "internal.h"
#include "lookup_common.h"

namespace infaas {

namespace {

constexpr int kGrpThreads = 1024;
constexpr int kGrpWaves = kGrpThreads / 64;
constexpr int kTile = kGroupTile;                    // queries per tile
constexpr int kTileRounds = kTile / (4 * kGrpThreads);   // a thread takes 4 consecutive queries per round
constexpr int32_t kUndecided = -2;                   // answer left to k_group_finish

__device__ __forceinline__ uint32_t acc_threshold16(int32_t min_acc, int32_t acc_base_m1)
{
    // keys are acc - acc_base + 1 in 1..65534, so a bound of 65535 already excludes every key
    const int32_t d = __builtin_elementwise_sub_sat(min_acc, acc_base_m1);
    return (uint32_t)(d < 1 ? 1 : (d > 65535 ? 65535 : d));
}

// ---------------------------------------------------------------- binning

// LDS: [group of every task, 16 bit][first task of every group][records per (wavefront, group)]
//      [the same as offsets into the tile][records per group][this workgroup's totals per group]
__global__ __launch_bounds__(kGrpThreads) void k_group_bin(TableView tv, IndexView ix, QueryView q, GroupScratch gs,
                                                           int32_t ntiles)
{
    extern __shared__ __align__(16) uint32_t lds[];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int G = (int)ix.num_groups, G1 = G + 1;
    publish_index_stats(tv);
   // group G: queries outside the table (answer -1)
    uint16_t *l_tg = (uint16_t *)lds;
    int32_t *l_t0 = (int32_t *)(lds + ((tv.T + 1) >> 1));
    uint32_t *l_cnt = (uint32_t *)(l_t0 + G1);          // [16][G1]
    uint32_t *l_off = l_cnt + kGrpWaves * G1;           // [16][G1]
    uint32_t *l_tot = l_off + kGrpWaves * G1;           // [G1 + 1] exclusive prefix of the groups' records in the tile
    uint32_t *l_sum = l_tot + G1 + 1;                   // [G1]
    for (int i = tid; i < tv.T; i += kGrpThreads) l_tg[i] = ix.task_group[i];
    for (int i = tid; i < G1; i += kGrpThreads) { l_t0[i] = ix.group_task0[i]; l_sum[i] = 0u; }
    if (blockIdx.x == 0)   // the statistics of this call are added up by k_group_finish
        for (int i = tid; i < gs.stat_blocks * kLookupStats; i += kGrpThreads) ix.stats[i] = 0u;
    const int32_t acc_base_m1 = tv.acc_base - 1;
    const bool aligned = ((((uintptr_t)q.task) | ((uintptr_t)q.slo) | ((uintptr_t)q.min_acc) | ((uintptr_t)q.bidx)) & 15u) == 0;
    // (barriers that order LDS traffic only: the previous tile's stores stay in flight across them)
    for (int32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        lds_barrier();   // tables ready; the previous tile's offsets have been read
        for (int i = tid; i < kGrpWaves * G1; i += kGrpThreads) l_cnt[i] = 0u;
        lds_barrier();
        const int64_t tile_base = (int64_t)tile * kTile;
        uint32_t w0[4 * kTileRounds], w1[4 * kTileRounds], gr[4 * kTileRounds];   // record words; group | rank << 8
#pragma unroll
        for (int r = 0; r < kTileRounds; ++r) {
            const int64_t i0 = tile_base + (int64_t)r * (4 * kGrpThreads) + tid * 4;
            int32_t tk[4], sl[4], am[4], bi[4];
            if (aligned && i0 + 4 <= q.n) {
                const v4i a = __builtin_nontemporal_load((const v4i *)(q.task + i0));
                const v4i b = __builtin_nontemporal_load((const v4i *)(q.slo + i0));
                const v4i c = __builtin_nontemporal_load((const v4i *)(q.min_acc + i0));
                const v4i d = __builtin_nontemporal_load((const v4i *)(q.bidx + i0));
                tk[0] = a.x; tk[1] = a.y; tk[2] = a.z; tk[3] = a.w; sl[0] = b.x; sl[1] = b.y; sl[2] = b.z; sl[3] = b.w;
                am[0] = c.x; am[1] = c.y; am[2] = c.z; am[3] = c.w; bi[0] = d.x; bi[1] = d.y; bi[2] = d.z; bi[3] = d.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool in = i0 + e < q.n;
                    tk[e] = in ? q.task[i0 + e] : -1; sl[e] = in ? q.slo[i0 + e] : 0;
                    am[e] = in ? q.min_acc[i0 + e] : 0; bi[e] = in ? q.bidx[i0 + e] : 0;
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool valid = ((uint32_t)tk[e] < (uint32_t)tv.T) & ((uint32_t)bi[e] < (uint32_t)tv.B) & (sl[e] >= 0);
                const uint32_t g = valid ? (uint32_t)l_tg[valid ? tk[e] : 0] : (uint32_t)G;
                const uint32_t slice = valid ? (uint32_t)(tk[e] - l_t0[g]) * (uint32_t)tv.B + (uint32_t)bi[e] : 0u;
                w0[4 * r + e] = (uint32_t)sl[e];
                w1[4 * r + e] = acc_threshold16(am[e], acc_base_m1) | (slice << 16);
                // rank among the wavefront's queries of the same group (any order will do: the
                // permutation is written out)
                const uint32_t rank = atomicAdd(&l_cnt[wave * G1 + g], 1u);
                gr[4 * r + e] = g | (rank << 8);
            }
        }
        lds_barrier();
        if (tid < G1) {   // records per group
            uint32_t t = 0;
            for (int w = 0; w < kGrpWaves; ++w) t += l_cnt[w * G1 + tid];
            l_sum[tid] += t;
            l_tot[tid + 1] = t;
        }
        lds_barrier();
        if (tid == 0) {   // exclusive prefix over the groups (at most 121 of them); entry G1: all records
            uint32_t run = 0;
            for (int g = 0; g < G1; ++g) { const uint32_t t = l_tot[g + 1]; l_tot[g] = run; run += t; }
            l_tot[G1] = run;
        }
        lds_barrier();
        for (int i = tid; i < kGrpWaves * G1; i += kGrpThreads) {   // where (wavefront, group) starts in the tile
            const int w = i / G1, g = i - w * G1;
            uint32_t at = l_tot[g];
            for (int v = 0; v < w; ++v) at += l_cnt[v * G1 + g];
            l_off[i] = at;
        }
        if (tid < G1) {   // the tile's run of every group: offset | length << 15
            const uint32_t start = l_tot[tid], len = l_tot[tid + 1] - start;
            gs.desc[(int64_t)tile * G1 + tid] = start | (len << 15);
        }
        lds_barrier();
#pragma unroll
        for (int r = 0; r < kTileRounds; ++r) {
            const int64_t i0 = tile_base + (int64_t)r * (4 * kGrpThreads) + tid * 4;
            uint32_t pos[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t g = gr[4 * r + e] & 0xFFu;
                pos[e] = l_off[wave * G1 + g] + (gr[4 * r + e] >> 8);
                const int64_t at = tile_base + pos[e];
                if (g < (uint32_t)G) gs.rec[at] = make_uint2(w0[4 * r + e], w1[4 * r + e]);
                else if (i0 + e < q.n) gs.res[at] = -1;
            }
            if (i0 + 4 <= q.n) {
                // (non-temporal like every access of the three kernels whose data is used once and is
                // coalesced: measured 5% on the whole path.  The records above are not: their 8-byte
                // stores rely on L2 to put lines together, and as non-temporal ones they take twice as long.)
                __builtin_nontemporal_store(((unsigned long long)(pos[2] | (pos[3] << 16)) << 32) | (pos[0] | (pos[1] << 16)),
                                            (unsigned long long *)(gs.perm + i0));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i0 + e < q.n) gs.perm[i0 + e] = (uint16_t)pos[e];
            }
        }
    }
    __syncthreads();
    if (tid < G && l_sum[tid]) atomicAdd(&gs.gcount[tid], l_sum[tid]);
}

// ---------------------------------------------------------------- lookup, group by group

// LDS: [control words][headers of the group's slices, and one of an empty slice][the group's region of the pool]
__global__ __launch_bounds__(kGrpThreads) void k_group_lookup(TableView tv, IndexView ix, GroupScratch gs, int32_t ntiles)
{
    extern __shared__ __align__(16) uint32_t lds_w[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int G1 = (int)ix.num_groups + 1;
    // The workgroups are dealt to the groups: one to every group that has records, the others in
    // proportion to the records (every workgroup works that out for itself, from the same counts).
    __shared__ int32_t s_plan[3];          // group of this workgroup, its number among the group's, how many those are
    __shared__ uint32_t s_count[128];
    for (int i = tid; i < G1 - 1; i += kGrpThreads) s_count[i] = gs.gcount[i];
    __syncthreads();
    if (tid == 0) {
        uint64_t total = 0;
        int32_t busy = 0;
        for (int i = 0; i < G1 - 1; ++i) { total += s_count[i]; busy += s_count[i] != 0u; }
        const int32_t spare = (int32_t)gridDim.x - busy;   // >= 0: there are at least as many workgroups as groups
        int32_t b = 0, mine = -1, rank = 0, n = 1;
        for (int i = 0; i < G1 - 1 && mine < 0; ++i) {
            const uint64_t c = s_count[i];
            if (c == 0) continue;
            const int32_t ni = 1 + (int32_t)((c * (uint64_t)spare) / total);
            if ((int32_t)blockIdx.x < b + ni) { mine = i; rank = (int32_t)blockIdx.x - b; n = ni; }
            b += ni;
        }
        s_plan[0] = mine; s_plan[1] = rank; s_plan[2] = n;
    }
    __syncthreads();
    const int32_t g = s_plan[0], wg_rank = s_plan[1], wg_n = s_plan[2];
    if (g < 0) return;
    const int32_t task0 = ix.group_task0[g], task1 = ix.group_task0[g + 1];
    const uint32_t s0 = (uint32_t)task0 * (uint32_t)tv.B, ns = (uint32_t)(task1 - task0) * (uint32_t)tv.B;
    const uint32_t hdr_bytes = ((ns + 1u) * kLdsHdrBytes + 15u) & ~15u;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(INFAAS_LDS uint32_t *)lds_w;
    const uint32_t lds_hdr0 = lds_base + kLdsCtrlBytes;
    const uint32_t rebase = lds_hdr0 + hdr_bytes;      // LDS address of the region's first byte
    const uint32_t region0 = (uint32_t)g * ix.region_bytes, step0 = (uint32_t)g * ix.group_step_cap;
    {
        // the group's region, as far as it has been handed out
        const uint32_t used = ix.gctrl[2 * g] < ix.region_bytes ? ix.gctrl[2 * g] : ix.region_bytes;
        const uint32_t nvec = (used + 15u) >> 4;
        const uint4 *gp = (const uint4 *)(ix.pool + region0);
        uint4 *lp = (uint4 *)(lds_w + ((kLdsCtrlBytes + hdr_bytes) >> 2));
        for (uint32_t i0 = tid; i0 < nvec; i0 += 4 * kGrpThreads) {   // four loads in flight per lane
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = gp[i0 + u * kGrpThreads < nvec ? i0 + u * kGrpThreads : 0];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * kGrpThreads < nvec) lp[i0 + u * kGrpThreads] = v[u];
        }
        // headers, rebased onto the LDS copy; a slice stored behind the regions, or without a body,
        // leaves its queries to k_group_finish; a slice without variants uses the region's own copy
        // of the empty body; entry ns stands for "no record"
        for (uint32_t s = tid; s <= ns; s += kGrpThreads) {
            uint4 h = s < ns ? ix.hdr[s0 + s] : make_uint4(0u, kEmptyHdrY, 0u, 0u);
            const bool parked = (h.y & kHdrPark) != 0u;
            const bool empty = !parked && h.x == 0u;
            const bool here = !parked && !empty && h.x + 4u >= region0 + kDummyBodyBytes && h.w <= region0 + ix.region_bytes &&
                              h.z >= step0 && h.z - step0 < 65536u;
            v2u l;
            l.x = ((here ? h.x - region0 : 0u) + rebase) | (h.y << kLdsAddrBits);   // high row bits above the address
            l.y = here ? ((h.y & 0xFFFF0000u) | (h.z - step0)) : (empty ? kEmptyHdrY : (kEmptyHdrY | kHdrPark | kHdrDeep));
            *(v2u *)(lds_w + (kLdsCtrlBytes / 4) + s * (kLdsHdrBytes / 4)) = l;
        }
    }
    if (tid < (int)(kLdsCtrlBytes / 4)) lds_w[tid] = 0u;
    __syncthreads();

    const uint32_t row_hi_mask = (1u << ix.row_hi_bits) - 1u;
    const uint32_t max_k = ix.ctrl[kCtlMaxK0];
    const int nit = 32 - __builtin_clz(max_k | 1u);    // <= 5
    const LdsMem lmem{};
    uint32_t &s_next = lds_w[2];
    // The wavefronts of the workgroup draw the group's runs (one per tile) from a counter in LDS; the
    // workgroups of a group take the tiles in turn.  The run after the current one is drawn, and its
    // descriptor requested, when the current one is started.
    auto draw = [&]() -> int32_t {
        uint32_t k = 0;
        if (lane == 0) k = atomicAdd(&s_next, 1u);
        k = (uint32_t)__builtin_amdgcn_readfirstlane((int)k);
        const int64_t tile = (int64_t)wg_rank + (int64_t)k * wg_n;
        return tile < ntiles ? (int32_t)tile : -1;
    };
    int32_t nxt_tile = draw();
    uint32_t nxt_desc = nxt_tile >= 0 ? gs.desc[(int64_t)nxt_tile * G1 + g] : 0u;
    int64_t run_base = 0;
    int32_t run_len = 0, run_at = 0;
    struct Unit {
        int64_t base;     // first record, or -1 when there is no unit left
        int32_t n;        // records (up to 256)
        uint2 rec[4];     // record k of a lane: 64 k + lane
    };
    auto fetch = [&](Unit &u) __attribute__((always_inline)) {
        while (run_at >= run_len) {
            if (nxt_tile < 0) { u.base = -1; u.n = 0; return; }
            run_base = (int64_t)nxt_tile * kTile + (nxt_desc & 0x7FFFu);
            run_len = (int32_t)(nxt_desc >> 15);
            run_at = 0;
            nxt_tile = draw();
            nxt_desc = nxt_tile >= 0 ? gs.desc[(int64_t)nxt_tile * G1 + g] : 0u;
        }
        u.base = run_base + run_at;
        u.n = run_len - run_at < 256 ? run_len - run_at : 256;
        run_at += 256;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t r = k * 64 + lane;
            const unsigned long long w = __builtin_nontemporal_load((const unsigned long long *)(gs.rec + u.base + (r < u.n ? r : 0)));
            u.rec[k] = make_uint2((uint32_t)w, (uint32_t)(w >> 32));
        }
    };
    // The answers of a unit are stored while the NEXT unit is answered, after its wait for memory:
    // rows fetched from step_row have arrived by then without anybody having waited for them.
    int64_t p_base = -1;
    int32_t p_n = 0, p_near[4], p_far[4];
    bool p_inl[4];
    auto store_pending = [&]() __attribute__((always_inline)) {
        if (p_base < 0) return;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (k * 64 + lane < p_n) __builtin_nontemporal_store(p_inl[k] ? p_near[k] : p_far[k], gs.res + p_base + k * 64 + lane);
    };
    auto answer = [&](const Unit &u) __attribute__((always_inline)) {
        uint32_t body[4], y[4], rec[4], keys[4], dd[4], lim[4], m[4], rbase[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool have = k * 64 + lane < u.n;
            const uint32_t s = have ? u.rec[k].y >> 16 : ns;
            const v2u h = lmem.ld64(lds_hdr0 + s * kLdsHdrBytes);
            body[k] = h.x & ((1u << kLdsAddrBits) - 1u); y[k] = h.y; rec[k] = h.y & 0xFFFFu;
            rbase[k] = h.x >> kLdsAddrBits;
            keys[k] = (y[k] >> kHdrK0Shift) & 0x3Fu;   // Re of the first body
            dd[k] = u.rec[k].y & 0xFFFFu;
            lim[k] = u.rec[k].x;
        }
        store_pending();
        search_bodies<4>(lmem, nit, body, keys, dd, lim, m);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool hit = m[k] != 0u;
            const uint32_t step = (uint32_t)__builtin_ctzg(m[k], -1);
            const bool inl = step < ix.hot_rows;   // its row sits in front of the body (low 16 bits) and in the header
            const uint32_t lo = lmem.ld16(inl ? body[k] - 2u * step : body[k], 2u);
            const uint32_t hi = (rbase[k] >> ((step * ix.row_hi_bits) & 31u)) & row_hi_mask;
            p_far[k] = ix.step_row[(hit && !inl) ? step0 + rec[k] + step : 0u];
            p_near[k] = hit ? (int32_t)((hi << 16) | lo) : ((int32_t)y[k] < 0 ? kUndecided : -1);   // (sign bit: a miss in
            p_inl[k] = inl || !hit;                                                                   //  the first body is not final)
        }
        p_base = u.base;
        p_n = u.n;
    };
    Unit ua, ub;
    fetch(ua);
    fetch(ub);
    for (;;) {   // two units in rotation: the records of the next one are under way while one is answered
        if (ua.base < 0) break;
        answer(ua);
        fetch(ua);
        if (ub.base < 0) break;
        answer(ub);
        fetch(ub);
    }
    store_pending();
}

// ---------------------------------------------------------------- back into query order

// Answer of one query from the index in global memory: first body, second body, and where the
// index is incomplete the rank-ordered scan of the slice (by the whole wavefront, one query at a
// time).  `active` lanes hold a query inside the table.  Counts what happened in st[1..4].
__device__ __forceinline__ int32_t resolve_from_memory(const TableView &tv, const IndexView &ix, bool active, int32_t task,
                                                       int32_t slo, int32_t min_acc, int32_t bidx, int nit, uint32_t (&st)[kLookupStats])
{
    const int lane = threadIdx.x & 63;
    const GlobalMem gmem{ix.pool};
    const uint32_t s = active ? (uint32_t)task * (uint32_t)tv.B + (uint32_t)bidx : (uint32_t)tv.S;
    const uint4 h = ix.hdr[s];
    const bool indexed = !(h.y & kHdrPark);
    const uint32_t keys0 = (h.y >> kHdrK0Shift) & 0x3Fu, keys1 = (h.y >> kHdrK1Shift) & 0x3Fu;
    const uint32_t dd[1] = {acc_threshold(min_acc, tv.acc_base - 1)}, lim[1] = {(uint32_t)slo};
    int32_t ans = -1;
    bool done = false;
    const bool need0 = active && indexed;
    if (__ballot(need0)) {
        const uint32_t bd[1] = {need0 ? h.x : 0u}, ks[1] = {need0 ? keys0 : 2u};
        uint32_t m[1];
        search_bodies<1>(gmem, nit, bd, ks, dd, lim, m);
        if (need0 && m[0]) { ans = ix.step_row[h.z + (uint32_t)__builtin_ctz(m[0])]; done = true; }
        st[2] += (uint32_t)__builtin_popcountll(__ballot(need0 && m[0]));
    }
    const bool need1 = active && indexed && keys1 != 0u && !done;
    if (__ballot(need1)) {
        const uint32_t bd[1] = {need1 ? h.x + body_bytes(keys0) : 0u}, ks[1] = {need1 ? keys1 : 2u};
        uint32_t m[1];
        search_bodies<1>(gmem, nit, bd, ks, dd, lim, m);
        if (need1 && m[0]) { ans = ix.step_row[h.z + kBodySteps + (uint32_t)__builtin_ctz(m[0])]; done = true; }
        st[1] += (uint32_t)__builtin_popcountll(__ballot(need1 && m[0]));
    }
    uint64_t todo = __ballot(active && !done && (!indexed || (h.y & kHdrTrunc)));
    st[3] += (uint32_t)__builtin_popcountll(todo);
    while (todo) {
        const int l = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int32_t t = __builtin_amdgcn_readlane(task, l), b = __builtin_amdgcn_readlane(bidx, l);
        const int32_t am = __builtin_amdgcn_readlane(min_acc, l);
        const uint32_t bound = (uint32_t)__builtin_amdgcn_readlane(slo, l);
        const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
        const int64_t col = (int64_t)b * tv.Vp + seg;
        int32_t found = -1;
        for (int32_t blk = 0; blk < L; blk += 64) {
            const int32_t pos = blk + lane;
            const bool ok = pos < L && tv.acc_r[col + pos] >= am && tv.tot_r[col + pos] <= bound;
            const uint64_t bm = __ballot(ok);
            if (bm) { found = blk + (int32_t)__builtin_ctzll(bm); break; }
        }
        if (lane == l) ans = found >= 0 ? tv.orig_r[col + found] : -1;
    }
    st[4] += (uint32_t)__builtin_popcountll(__ballot(active && ans < 0));
    return ans;
}

__global__ __launch_bounds__(kGrpThreads) void k_group_finish(TableView tv, IndexView ix, QueryView q, GroupScratch gs,
                                                              int32_t ntiles)
{
    __shared__ int32_t l_res[kTile];
    __shared__ uint32_t l_st[kLookupStats];
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t max_k = ix.ctrl[kCtlMaxK0];
    const int nit = 32 - __builtin_clz(max_k | 1u);
    uint32_t st[kLookupStats] = {0u, 0u, 0u, 0u, 0u};
    if (tid < kLookupStats) l_st[tid] = 0u;
    if (blockIdx.x == 0 && tid <= (int)ix.num_groups) gs.gcount[tid] = 0u;   // for the next call's binning
    const bool aligned = (((uintptr_t)q.out) & 15u) == 0;
    // The barriers order LDS traffic only, so a tile's stores, and the loads of the next tile's answers,
    // stay in flight across them.
    constexpr int kResRounds = kTile / (4 * kGrpThreads);
    v4i nxt[kResRounds];                      // the answers of the tile that comes next, in binned order
    unsigned long long nxt_pos[kTileRounds];  // and where each of its queries' answers is, four 16-bit positions a word
    auto request = [&](int32_t tile) {
#pragma unroll
        for (int r = 0; r < kResRounds; ++r)
            nxt[r] = __builtin_nontemporal_load((const v4i *)(gs.res + (int64_t)tile * kTile + r * 4 * kGrpThreads + tid * 4));
#pragma unroll
        for (int r = 0; r < kTileRounds; ++r) {
            const int64_t i0 = (int64_t)tile * kTile + (int64_t)r * (4 * kGrpThreads) + tid * 4;
            if (i0 + 4 <= q.n) {
                nxt_pos[r] = __builtin_nontemporal_load((const unsigned long long *)(gs.perm + i0));
            } else {
                nxt_pos[r] = 0ull;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i0 + e < q.n) nxt_pos[r] |= (unsigned long long)gs.perm[i0 + e] << (16 * e);
            }
        }
    };
    if ((int32_t)blockIdx.x < ntiles) request((int32_t)blockIdx.x);
    for (int32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t tile_base = (int64_t)tile * kTile;
        lds_barrier();   // the previous tile's answers have been read
#pragma unroll
        for (int r = 0; r < kResRounds; ++r) *(v4i *)&l_res[r * 4 * kGrpThreads + tid * 4] = nxt[r];
        uint32_t pos_all[kTileRounds][4];
#pragma unroll
        for (int r = 0; r < kTileRounds; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) pos_all[r][e] = (uint32_t)(nxt_pos[r] >> (16 * e)) & 0xFFFFu;
        lds_barrier();
        if (tile + (int32_t)gridDim.x < ntiles) request(tile + (int32_t)gridDim.x);
#pragma unroll
        for (int r = 0; r < kTileRounds; ++r) {
            const int64_t i0 = tile_base + (int64_t)r * (4 * kGrpThreads) + tid * 4;
            const uint32_t *pos = pos_all[r];
            int32_t a[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] = i0 + e < q.n ? l_res[pos[e] & (kTile - 1)] : -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // (rare) queries the group's LDS copy could not decide
                const bool open = a[e] == kUndecided;
                const uint64_t any = __ballot(open);
                if (any) {
                    st[0] += (uint32_t)__builtin_popcountll(any);
                    const int64_t i = open ? i0 + e : 0;
                    const int32_t v = resolve_from_memory(tv, ix, open, q.task[i], q.slo[i], q.min_acc[i], q.bidx[i], nit, st);
                    if (open) a[e] = v;
                }
            }
            if (aligned && i0 + 4 <= q.n) {
                const v4i v = {a[0], a[1], a[2], a[3]};
                __builtin_nontemporal_store(v, (v4i *)(q.out + i0));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i0 + e < q.n) q.out[i0 + e] = a[e];
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < kLookupStats; ++i)
            if (st[i]) atomicAdd(&l_st[i], st[i]);
    }
    __syncthreads();
    if (tid < kLookupStats && l_st[tid]) atomicAdd(&ix.stats[(blockIdx.x % (unsigned)gs.stat_blocks) * kLookupStats + tid], l_st[tid]);
}

}  // namespace

// ---------------------------------------------------------------- launchers

size_t group_bin_lds_bytes(int32_t T, int32_t G)
{
    const size_t G1 = (size_t)G + 1;
    return 4 * (((size_t)T + 1) / 2 + G1 + 2 * kGrpWaves * G1 + (G1 + 1) + G1) + 16;
}

hipError_t launch_group_bin(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                            int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    const int32_t ntiles = (q.n + kTile - 1) / kTile;
    const int blocks = ntiles < num_cus ? ntiles : num_cus;
    return launch_kernel(ev, k_group_bin, dim3((unsigned)blocks), dim3(kGrpThreads), group_bin_lds_bytes(tv.T, (int32_t)ix.num_groups),
                         st, tv, ix, q, gs, ntiles);
}

hipError_t launch_group_lookup(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                               int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    const int32_t ntiles = (q.n + kTile - 1) / kTile;
    // control words, the headers of the largest group, a region
    const uint32_t lds = kLdsCtrlBytes + ((((uint32_t)gs.max_group_slices + 1u) * kLdsHdrBytes + 15u) & ~15u) + ix.region_bytes;
    hipError_t e = hipFuncSetAttribute((const void *)k_group_lookup, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    return launch_kernel(ev, k_group_lookup, dim3((unsigned)num_cus), dim3(kGrpThreads), lds, st, tv, ix, gs, ntiles);
}

hipError_t launch_group_finish(const TableView &tv, const IndexView &ix, const QueryView &q, const GroupScratch &gs,
                               int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    const int32_t ntiles = (q.n + kTile - 1) / kTile;
    // one workgroup per compute unit (its registers leave no room for a second): the next tile's answers
    // and positions are requested while the current tile is written
    const int blocks = ntiles < num_cus ? ntiles : num_cus;
    return launch_kernel(ev, k_group_finish, dim3((unsigned)blocks), dim3(kGrpThreads), 0, st, tv, ix, q, gs, ntiles);
}

}  // namespace infaas
