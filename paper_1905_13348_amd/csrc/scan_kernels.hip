// Exhaustive-scan engine of the variant selection (Section 4.1 of the INFaaS paper; the
// brute-force search that Section 6.4 uses as its yardstick), written for gfx950.
//
//   histogram -> plan -> scatter : bucket the queries by (task, batch) slice
//   scan (LDS)                   : a workgroup stages one slice once and answers a tile of
//                                  that slice's queries; each wavefront filters 256 variants
//                                  per step for 4 queries and min-reduces the survivors
//   scan (wide) + finish         : slices larger than the LDS budget are cut into chunks that
//                                  different workgroups scan; partial minima meet in a
//                                  device-wide atomicMin per query
//
// The lexicographic key (cost, profiled latency, caller row) of every variant is replaced by
// its rank inside its slice, computed once when the table is loaded, so the argmin runs on
// 32-bit integers and its result is unique.
#include "internal.h"
#include "lookup_common.h"

namespace infaas {

namespace {

constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kQueriesPerWavePass = 4;
constexpr int kScatterThreads = 256;
constexpr int kScatterPerThread = 8;

__device__ __forceinline__ int32_t slice_of(const TableView &tv, int32_t task, int32_t slo,
                                            int32_t bidx)
{
    if ((uint32_t)task >= (uint32_t)tv.T || (uint32_t)bidx >= (uint32_t)tv.B || slo < 0)
        return -1;
    if (tv.seg_len[task] == 0)
        return -1;
    return task * tv.B + bidx;
}

// Minimum over the 64 lanes of a wavefront, returned wave-uniform.
// Four DPP steps make every lane of a 16-lane row hold the row minimum; the four row
// minima are then read from one lane of each row.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    uint32_t o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    v = v < o ? v : o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    v = v < o ? v : o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);  // row_half_mirror
    v = v < o ? v : o;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);  // row_mirror
    v = v < o ? v : o;
    uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
    uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
    uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    r0 = r0 < r1 ? r0 : r1;
    r2 = r2 < r3 ? r2 : r3;
    return r0 < r2 ? r0 : r2;
}

__device__ __forceinline__ int32_t wave_incl_scan(int32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int32_t o = __shfl_up(v, d, 64);
        if (lane >= d)
            v += o;
    }
    return v;
}

// ---------------------------------------------------------------- load update

// Rewinds the allocator of the index and clears its statistics (the index is rebuilt after every
// report): thread 0 the counters of the pool as a whole, threads 0 .. groups - 1 those of the groups'
// regions (every region begins with the dummy body; entry 0 of step_row, in group 0's part, is unused).
__device__ __forceinline__ void rewind_index(const IndexView &ix, int64_t tid)
{
    if (!ix.ctrl) return;
    if (tid == 0) {
        ix.ctrl[kCtlPool] = ix.ctrl[kCtlPool0];
        ix.ctrl[kCtlSteps] = ix.ctrl[kCtlSteps0];
        ix.ctrl[kCtlEpoch] = (ix.ctrl[kCtlEpoch] + 1u) & 0xFFFu;
        ix.ctrl[kCtlMaxK0] = 1;
        ix.ctrl[kCtlTrunc] = 0;
        ix.ctrl[kCtlNoBody] = 0;
        ix.ctrl[kCtlMaxK] = 0;
    }
    if (ix.num_groups > 1 && tid < (int64_t)ix.num_groups) {
        ix.gctrl[2 * tid] = kDummyBodyBytes;
        ix.gctrl[2 * tid + 1] = tid == 0 ? 1u : 0u;
    }
}

// One thread per (update, batch size): the queue itself, and latency-plus-queue of the variant's
// entry in each rank-ordered column.  Thread 0 also rewinds the index allocator, because the
// index is rebuilt after every load report.
__global__ __launch_bounds__(256) void k_update_load(TableView tv, int32_t n,
                                                     const int32_t *__restrict__ idx,
                                                     const int32_t *__restrict__ val,
                                                     IndexView ix)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    rewind_index(ix, tid);
    if (tid >= (int64_t)n * tv.B)
        return;
    const int32_t i = (int32_t)(tid / tv.B), b = (int32_t)(tid - (int64_t)i * tv.B);
    const int32_t v = idx[i];
    const int32_t x = val[i];
    if ((uint32_t)v >= (uint32_t)tv.V || x < 0)
        return;
    const int32_t slot = tv.slot_of[v];
    if (b == 0) tv.queue[slot] = x;
    const int64_t g = (int64_t)b * tv.Vp + tv.gpos[(int64_t)b * tv.Vp + slot];
    const bool masked = tv.state && tv.state[slot] != tv.want_state;
    tv.tot_r[g] = masked ? 0xFFFFFFFFu : (uint32_t)tv.lat_r[g] + (uint32_t)x;
}

// One thread per (report entry, batch size): the state itself, and the masked or restored entry
// of the variant in each rank-ordered column.  idx null: entry i is row i.  Rewinds the index
// allocator like a load update, because the index is rebuilt afterwards.
__global__ __launch_bounds__(256) void k_update_state(TableView tv, int32_t n,
                                                      const int32_t *__restrict__ idx,
                                                      const int32_t *__restrict__ val,
                                                      IndexView ix)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    rewind_index(ix, tid);
    if (tid >= (int64_t)n * tv.B)
        return;
    const int32_t i = (int32_t)(tid / tv.B), b = (int32_t)(tid - (int64_t)i * tv.B);
    const int32_t v = idx ? idx[i] : i;
    const int32_t x = val[i];
    if ((uint32_t)v >= (uint32_t)tv.V || (uint32_t)x > 3u)
        return;
    const int32_t slot = tv.slot_of[v];
    if (b == 0) tv.state[slot] = x;
    const int64_t g = (int64_t)b * tv.Vp + tv.gpos[(int64_t)b * tv.Vp + slot];
    const bool masked = x != tv.want_state;
    tv.tot_r[g] = masked ? 0xFFFFFFFFu : (uint32_t)tv.lat_r[g] + (uint32_t)tv.queue[slot];
    tv.acc_r[g] = masked ? tv.acc_base : tv.acc[slot];
}

// ---------------------------------------------------------------- bucketing

template <bool kLds>
__global__ __launch_bounds__(256) void k_histogram(TableView tv, QueryView q,
                                                   int32_t *__restrict__ cnt)
{
    extern __shared__ int32_t lds_hist[];
    const int tid = threadIdx.x;
    publish_index_stats(tv);
    if (kLds) {
        for (int i = tid; i < tv.S; i += 256) lds_hist[i] = 0;
        __syncthreads();
    }
    int64_t per = ((int64_t)q.n + gridDim.x - 1) / gridDim.x;
    int64_t begin = (int64_t)blockIdx.x * per;
    int64_t end = begin + per < (int64_t)q.n ? begin + per : (int64_t)q.n;
    for (int64_t i = begin + tid; i < end; i += 256) {
        int32_t s = slice_of(tv, q.task[i], q.slo[i], q.bidx[i]);
        if (s >= 0) {
            if (kLds) atomicAdd(&lds_hist[s], 1);
            else atomicAdd(&cnt[s], 1);
        }
    }
    if (kLds) {
        __syncthreads();
        for (int i = tid; i < tv.S; i += 256) {
            int32_t c = lds_hist[i];
            if (c) atomicAdd(&cnt[i], c);
        }
    }
}

// One workgroup: exclusive prefix sums of (queries, LDS tiles, wide work items) per slice.
// Consumes cnt and leaves it zero for the next call.
__global__ __launch_bounds__(1024) void k_plan(TableView tv, ScanScratch sc)
{
    __shared__ int32_t wsum[3][16];
    __shared__ int32_t carry[3];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid < 3) carry[tid] = 0;
    __syncthreads();
    for (int32_t base = 0; base < tv.S; base += 1024) {
        int32_t s = base + tid;
        int32_t v[3] = {0, 0, 0};
        if (s < tv.S) {
            int32_t c = sc.cnt[s];
            sc.cnt[s] = 0;
            int32_t L = tv.seg_len[s / tv.B];
            int32_t tiles = (c + kQueriesPerTile - 1) / kQueriesPerTile;
            v[0] = c;
            if (L > tv.lds_limit) v[2] = tiles * ((L + tv.lds_limit - 1) / tv.lds_limit);
            else v[1] = tiles;
        }
        int32_t inc[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            inc[k] = wave_incl_scan(v[k]);
            if (lane == 63) wsum[k][w] = inc[k];
        }
        __syncthreads();
        if (tid < 3) {  // serial exclusive scan of the 16 wave totals
            int32_t run = 0;
            for (int j = 0; j < 16; ++j) {
                int32_t x = wsum[tid][j];
                wsum[tid][j] = run;
                run += x;
            }
        }
        __syncthreads();
        int32_t ex[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) ex[k] = carry[k] + wsum[k][w] + inc[k] - v[k];
        if (s < tv.S) {
            sc.bucket_off[s] = ex[0];
            sc.cursor[s] = ex[0];
            sc.tile_off[s] = ex[1];
            sc.wide_off[s] = ex[2];
        }
        __syncthreads();
        if (tid == 1023) {
#pragma unroll
            for (int k = 0; k < 3; ++k) carry[k] = ex[k] + v[k];
        }
        __syncthreads();
    }
    if (tid == 0) {
        sc.bucket_off[tv.S] = carry[0];
        sc.tile_off[tv.S] = carry[1];
        sc.wide_off[tv.S] = carry[2];
        sc.counters[0] = 0;
        sc.counters[1] = 0;
    }
}

template <bool kLds>
__global__ __launch_bounds__(kScatterThreads) void k_scatter(TableView tv, QueryView q,
                                                             ScanScratch sc, int init_best)
{
    extern __shared__ int32_t lds_cnt[];
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * (kScatterThreads * kScatterPerThread);
    if (kLds) {
        for (int i = tid; i < tv.S; i += kScatterThreads) lds_cnt[i] = 0;
        __syncthreads();
    }
    int32_t sl[kScatterPerThread], rk[kScatterPerThread], slo[kScatterPerThread],
        am[kScatterPerThread];
#pragma unroll
    for (int k = 0; k < kScatterPerThread; ++k) {
        int64_t i = base + k * kScatterThreads + tid;
        sl[k] = -1;
        rk[k] = 0;
        slo[k] = 0;
        am[k] = 0;
        if (i < q.n) {
            slo[k] = q.slo[i];
            am[k] = q.min_acc[i];
            int32_t s = slice_of(tv, q.task[i], slo[k], q.bidx[i]);
            sl[k] = s;
            if (s < 0) q.out[i] = -1;
            else rk[k] = kLds ? atomicAdd(&lds_cnt[s], 1) : atomicAdd(&sc.cursor[s], 1);
        }
    }
    if (kLds) {
        __syncthreads();
        for (int i = tid; i < tv.S; i += kScatterThreads) {
            int32_t c = lds_cnt[i];
            if (c) lds_cnt[i] = atomicAdd(&sc.cursor[i], c);
        }
        __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < kScatterPerThread; ++k) {
        if (sl[k] < 0) continue;
        int64_t i = base + k * kScatterThreads + tid;
        int32_t pos = rk[k] + (kLds ? lds_cnt[sl[k]] : 0);
        sc.recs[pos] = make_int4(slo[k], am[k], (int32_t)i, sl[k]);
        if (init_best) sc.best[pos] = kNoRank;
    }
}

// ---------------------------------------------------------------- scan

// Largest s in [0, n-1) with off[s] <= x, for a non-decreasing off[0..n-1] with off[0] = 0.
__device__ __forceinline__ int32_t find_owner(const int32_t *__restrict__ off, int32_t n,
                                              int32_t x)
{
    int32_t lo = 0, hi = n;  // invariant: off[lo] <= x, (hi == n or off[hi] > x)
    while (hi - lo > 1) {
        int32_t mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

template <bool kWide>
__global__ __launch_bounds__(kScanThreads) void k_scan(TableView tv, QueryView q, ScanScratch sc,
                                                       int32_t lds_entries)
{
    extern __shared__ int32_t lds_raw[];
    int32_t *l_acc = lds_raw;
    uint32_t *l_tot = (uint32_t *)(lds_raw + lds_entries);
    uint32_t *l_rank = (uint32_t *)(lds_raw + 2 * lds_entries);
    __shared__ int32_t s_item;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t *off = kWide ? sc.wide_off : sc.tile_off;
    const int32_t total = off[tv.S];

    for (;;) {
        if (tid == 0) s_item = atomicAdd(&sc.counters[kWide ? 1 : 0], 1);
        __syncthreads();
        const int32_t item = s_item;
        __syncthreads();
        if (item >= total) break;

        const int32_t s = find_owner(off, tv.S + 1, item);
        const int32_t t = s / tv.B, b = s - t * tv.B;
        const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
        int32_t local = item - off[s];
        int32_t tile = local, c_begin = 0, c_end = L;
        if (kWide) {
            int32_t nch = (L + tv.lds_limit - 1) / tv.lds_limit;
            tile = local / nch;
            int32_t ch = local - tile * nch;
            c_begin = ch * tv.lds_limit;
            c_end = c_begin + tv.lds_limit < L ? c_begin + tv.lds_limit : L;
        }
        const int32_t first = sc.bucket_off[s] + tile * kQueriesPerTile;
        int32_t count = sc.bucket_off[s + 1] - first;
        if (count > kQueriesPerTile) count = kQueriesPerTile;

        // stage rows [c_begin, c_end) of the slice, 4 per 128-bit load, padded to 256 entries
        const int32_t len4 = (c_end - c_begin + 3) & ~3;           // rows present incl. row padding
        const int32_t lenp = (c_end - c_begin + 255) & ~255;       // entries the scan loop visits
        const int64_t col = (int64_t)b * tv.Vp + seg + c_begin;
        for (int32_t i = tid * 4; i < lenp; i += kScanThreads * 4) {
            int4 a = make_int4(INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN);
            uint4 tt = make_uint4(~0u, ~0u, ~0u, ~0u);
            uint4 rr = tt;
            if (i < len4) {
                a = *(const int4 *)(tv.acc + seg + c_begin + i);
                int4 qv = *(const int4 *)(tv.queue + seg + c_begin + i);
                int4 lv = *(const int4 *)(tv.lat + col + i);
                rr = *(const uint4 *)(tv.rank + col + i);
                tt = make_uint4((uint32_t)lv.x + (uint32_t)qv.x, (uint32_t)lv.y + (uint32_t)qv.y,
                                (uint32_t)lv.z + (uint32_t)qv.z, (uint32_t)lv.w + (uint32_t)qv.w);
            }
            *(int4 *)(l_acc + i) = a;
            *(uint4 *)(l_tot + i) = tt;
            *(uint4 *)(l_rank + i) = rr;
        }
        __syncthreads();

        for (int32_t qi = wave * kQueriesPerWavePass; qi < count;
             qi += kScanWaves * kQueriesPerWavePass) {
            int32_t slo[kQueriesPerWavePass], am[kQueriesPerWavePass], qid[kQueriesPerWavePass];
            uint32_t best[kQueriesPerWavePass];
#pragma unroll
            for (int k = 0; k < kQueriesPerWavePass; ++k) {
                int32_t j = qi + k < count ? qi + k : count - 1;
                int4 r = sc.recs[first + j];
                slo[k] = __builtin_amdgcn_readfirstlane(r.x);
                am[k] = __builtin_amdgcn_readfirstlane(r.y);
                qid[k] = __builtin_amdgcn_readfirstlane(r.z);
                best[k] = kNoRank;
            }
            for (int32_t i = lane * 4; i < lenp; i += 256) {
                const int4 a = *(const int4 *)(l_acc + i);
                const uint4 tt = *(const uint4 *)(l_tot + i);
                const uint4 rr = *(const uint4 *)(l_rank + i);
#pragma unroll
                for (int k = 0; k < kQueriesPerWavePass; ++k) {
                    const uint32_t lim = (uint32_t)slo[k];
                    uint32_t c0 = (a.x >= am[k] && tt.x <= lim) ? rr.x : kNoRank;
                    uint32_t c1 = (a.y >= am[k] && tt.y <= lim) ? rr.y : kNoRank;
                    uint32_t c2 = (a.z >= am[k] && tt.z <= lim) ? rr.z : kNoRank;
                    uint32_t c3 = (a.w >= am[k] && tt.w <= lim) ? rr.w : kNoRank;
                    c0 = c0 < c1 ? c0 : c1;
                    c2 = c2 < c3 ? c2 : c3;
                    c0 = c0 < c2 ? c0 : c2;
                    best[k] = best[k] < c0 ? best[k] : c0;
                }
            }
#pragma unroll
            for (int k = 0; k < kQueriesPerWavePass; ++k) {
                const uint32_t m = wave_min_u32(best[k]);
                if (lane == k && qi + k < count) {
                    if (kWide) {
                        if (m != kNoRank) atomicMin(&sc.best[first + qi + k], m);
                    } else {
                        int32_t ans = -1;
                        if (m != kNoRank)
                            ans = tv.orig[seg + tv.perm[(int64_t)b * tv.Vp + seg + m]];
                        q.out[qid[k]] = ans;
                    }
                }
            }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void k_finish_wide(TableView tv, QueryView q, ScanScratch sc)
{
    const int32_t total = sc.bucket_off[tv.S];
    for (int32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < total;
         p += gridDim.x * blockDim.x) {
        int4 r = sc.recs[p];
        int32_t s = r.w;
        int32_t t = s / tv.B, b = s - t * tv.B;
        if (tv.seg_len[t] <= tv.lds_limit) continue;
        uint32_t m = sc.best[p];
        int32_t ans = -1;
        if (m != kNoRank) {
            int32_t seg = tv.seg_off[t];
            ans = tv.orig[seg + tv.perm[(int64_t)b * tv.Vp + seg + m]];
        }
        q.out[r.z] = ans;
    }
}

// The closest-variant suggestion (Section 4.1, last step of Case I) for a handle without the
// staircase index: q.out holds the selection already; q.closest becomes the selection where there is
// one, else the variant of the query's slice that comes closest, found by the whole wavefront, one
// such query at a time.  Exhaustive like the engine it belongs to.
__global__ __launch_bounds__(256) void k_closest_scan(TableView tv, QueryView q)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6, nwaves = (int64_t)gridDim.x * 4;
    for (int64_t base = wave * 64; base < q.n; base += nwaves * 64) {
        const int64_t i = base + lane;
        const bool in = i < q.n;
        const int32_t sel = in ? q.out[i] : 0;
        const int32_t task = in ? q.task[i] : -1, bidx = in ? q.bidx[i] : -1;
        const int32_t slo = in ? q.slo[i] : 0, min_acc = in ? q.min_acc[i] : 0;
        const bool inside = in && (uint32_t)task < (uint32_t)tv.T && (uint32_t)bidx < (uint32_t)tv.B;
        int32_t sug = sel;   // (a query outside the table has no selection and gets no suggestion)
        uint64_t rest = __ballot(inside && sel < 0);
        while (rest) {
            const int l = __builtin_ctzll(rest);
            rest &= rest - 1;
            const int32_t t = __builtin_amdgcn_readlane(task, l), b = __builtin_amdgcn_readlane(bidx, l);
            const int64_t am = __builtin_amdgcn_readlane(min_acc, l), bound = __builtin_amdgcn_readlane(slo, l);
            const int32_t found = closest_by_scan(tv, t, b, am, bound, lane);
            if (lane == l) sug = found;
        }
        if (in) q.closest[i] = sug;
    }
}

}  // namespace

// ---------------------------------------------------------------- launchers

hipError_t launch_update_load(const TableView &tv, int32_t n, const int32_t *idx,
                              const int32_t *val, const IndexView *index, hipStream_t st, const LaunchEvents *ev)
{
    if (n <= 0) return hipSuccess;
    const int64_t threads = (int64_t)n * tv.B;   // (n >= 1: at least 256 threads, more than there are groups)
    return launch_kernel(ev, k_update_load, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, tv, n, idx, val,
                         index ? *index : IndexView{});
}

hipError_t launch_update_state(const TableView &tv, int32_t n, const int32_t *idx,
                               const int32_t *val, const IndexView *index, hipStream_t st, const LaunchEvents *ev)
{
    if (n <= 0) return hipSuccess;
    const int64_t threads = (int64_t)n * tv.B;
    return launch_kernel(ev, k_update_state, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, tv, n, idx, val,
                         index ? *index : IndexView{});
}

hipError_t launch_histogram(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            hipStream_t st, const LaunchEvents *ev)
{
    int blocks = (int)((q.n + 16383) / 16384);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    if (tv.S <= kLdsHistMaxSlices)
        return launch_kernel(ev, k_histogram<true>, dim3((unsigned)blocks), dim3(256), (size_t)tv.S * 4, st, tv, q, sc.cnt);
    else
        return launch_kernel(ev, k_histogram<false>, dim3((unsigned)blocks), dim3(256), 0, st, tv, q, sc.cnt);
}

hipError_t launch_plan(const TableView &tv, const ScanScratch &sc, hipStream_t st, const LaunchEvents *ev)
{
    return launch_kernel(ev, k_plan, dim3(1), dim3(1024), 0, st, tv, sc);
}

hipError_t launch_scatter(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                          bool init_best, hipStream_t st, const LaunchEvents *ev)
{
    const int per_block = kScatterThreads * kScatterPerThread;
    int blocks = (q.n + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (tv.S <= kLdsHistMaxSlices)
        return launch_kernel(ev, k_scatter<true>, dim3((unsigned)blocks), dim3((unsigned)kScatterThreads), (size_t)tv.S * 4, st, tv, q, sc, init_best);
    else
        return launch_kernel(ev, k_scatter<false>, dim3((unsigned)blocks), dim3((unsigned)kScatterThreads), 0, st, tv, q, sc, init_best);
}

static int scan_blocks(int num_cus, size_t lds_bytes)
{
    int per_cu = (int)((160 * 1024) / (lds_bytes + 512));
    if (per_cu > 8) per_cu = 8;
    if (per_cu < 1) per_cu = 1;
    return num_cus * per_cu;
}

hipError_t launch_scan_lds(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                           int32_t max_lds_segment, int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    int32_t entries = (max_lds_segment + 255) & ~255;
    if (entries < 256) entries = 256;
    size_t lds = (size_t)entries * 12;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)k_scan<false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return launch_kernel(ev, k_scan<false>, dim3((unsigned)(scan_blocks(num_cus, lds))), dim3((unsigned)kScanThreads), lds, st, tv, q, sc, entries);
}

hipError_t launch_scan_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                            int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    int32_t entries = (tv.lds_limit + 255) & ~255;
    size_t lds = (size_t)entries * 12;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)k_scan<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return launch_kernel(ev, k_scan<true>, dim3((unsigned)(scan_blocks(num_cus, lds))), dim3((unsigned)kScanThreads), lds, st, tv, q, sc, entries);
}

hipError_t launch_finish_wide(const TableView &tv, const QueryView &q, const ScanScratch &sc,
                              hipStream_t st, const LaunchEvents *ev)
{
    int blocks = (q.n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    return launch_kernel(ev, k_finish_wide, dim3((unsigned)blocks), dim3(256), 0, st, tv, q, sc);
}

hipError_t launch_closest_scan(const TableView &tv, const QueryView &q, int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    if (q.n <= 0) return hipSuccess;
    const int64_t want = ((int64_t)q.n + 255) / 256, most = (int64_t)num_cus * 8;
    return launch_kernel(ev, k_closest_scan, dim3((unsigned)(want < most ? want : most)), dim3(256), 0, st, tv, q);
}

}  // namespace infaas
