// Staircase index of the variant selection (Section 4.1 of the INFaaS paper): the same
// answers as the exhaustive scan, reached through a per-slice structure that keeps only the
// variants that can ever be chosen.  The paper's own controller answers in milliseconds where
// its brute-force search needs ~100 ms because its metadata store keeps sorted sets
// (Sections 5 and 6.4); this is the exact, batched GPU counterpart of that idea.
//
//   k_index_build  : one wavefront per (task, batch) slice walks the slice in rank order and
//                    keeps the "steps" (variants not dominated by a cheaper one), then writes
//                    sorted keys and bit sets for them (layout: see BodyLayout)
//   k_index_select : one lane per query.  The whole index is mirrored in LDS; a query costs two
//                    binary searches in LDS, two bit-set reads, one AND and one count-trailing-
//                    zeros.  Queries it cannot decide from LDS (slice not resident, or staircase
//                    truncated and no step fits) are parked and finished by the same workgroup:
//                    first from the index copy in global memory, then by a wavefront-wide scan of
//                    the rank-ordered slice that stops at the first feasible variant.
#include "internal.h"

namespace infaas {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kSelThreads = 1024;
constexpr int kPerThread = 4;
static_assert(kSelThreads * kPerThread == kIndexTile, "tile = threads x queries per thread");

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---------------------------------------------------------------- build

__global__ __launch_bounds__(64) void k_index_build(TableView tv, IndexView ix)
{
    const int32_t s = blockIdx.x;
    if (s >= tv.S) return;
    const int lane = threadIdx.x;
    const int32_t t = s / tv.B, b = s - t * tv.B;
    const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
    const BodyLayout empty(0, false);
    if (L == 0) {  // no variants: the K = 0 dummy body at offset 0 answers "nothing feasible"
        if (lane == 0) {
            ix.hdr[2 * s] = make_uint4(0u - 2u, empty.o_tot - 4u, empty.o_ea - 4u, empty.o_es - 4u);
            ix.hdr[2 * s + 1] = make_uint4(1u | kHdrIndexed, 0u, 0u, empty.size);
        }
        return;
    }
    const int32_t *__restrict__ accc = tv.acc_r + (int64_t)b * tv.Vp + seg;
    const uint32_t *__restrict__ totc = tv.tot_r + (int64_t)b * tv.Vp + seg;

    // ---- phase A: the steps, in rank order; lane j keeps step j
    int32_t K = 0;
    bool trunc = false;
    int32_t st_acc = 0, st_pos = 0;
    uint32_t st_tot = 0;
    int32_t a_nx = lane < L ? accc[lane] : INT32_MIN;
    uint32_t t_nx = lane < L ? totc[lane] : 0xFFFFFFFFu;
    for (int32_t blk = 0; blk < L && !trunc; blk += 64) {
        const int32_t a = a_nx;
        const uint32_t tt = t_nx;
        bool alive = blk + lane < L;
        const int32_t nx = blk + 64 + lane;
        a_nx = nx < L ? accc[nx] : INT32_MIN;
        t_nx = nx < L ? totc[nx] : 0xFFFFFFFFu;
        for (int32_t j = 0; j < K; ++j) {
            const int32_t aj = __builtin_amdgcn_readlane(st_acc, j);
            const uint32_t tj = (uint32_t)__builtin_amdgcn_readlane((int)st_tot, j);
            alive = alive && !(aj >= a && tj <= tt);
            if ((j & 3) == 3 && __ballot(alive) == 0) break;
        }
        uint64_t mask = __ballot(alive);
        while (mask) {
            if (K == kIndexCap) { trunc = true; break; }
            const int l = __builtin_ctzll(mask);
            const int32_t al = __builtin_amdgcn_readlane(a, l);
            const uint32_t tl = (uint32_t)__builtin_amdgcn_readlane((int)tt, l);
            if (lane == K) { st_acc = al; st_tot = tl; st_pos = blk + l; }
            K += 1;
            alive = alive && !(al >= a && tl <= tt);   // also retires lane l itself
            mask = __ballot(alive);
        }
    }

    // ---- phase B: sorted keys and bit sets
    int32_t lo = __builtin_amdgcn_readlane(st_acc, 0), hi = lo;
    for (int32_t j = 1; j < K; ++j) {
        const int32_t aj = __builtin_amdgcn_readlane(st_acc, j);
        lo = aj < lo ? aj : lo;
        hi = aj > hi ? aj : hi;
    }
    const bool wide = K > 32;
    const BodyLayout lay((uint32_t)K, wide);
    uint32_t off = 0, rec = 0;
    if (lane == 0) {
        off = atomicAdd(&ix.ctrl[0], lay.size);
        rec = atomicAdd(&ix.ctrl[1], (uint32_t)K);
    }
    off = (uint32_t)__builtin_amdgcn_readfirstlane((int)off);
    rec = (uint32_t)__builtin_amdgcn_readfirstlane((int)rec);
    const bool fits = (uint64_t)off + lay.size <= ix.pool_bytes && (uint64_t)rec + K <= ix.step_cap &&
                      (int64_t)hi - (int64_t)lo <= 65533;
    if (!fits) {  // no body: every query of this slice goes to the rank-ordered scan
        if (lane == 0) {
            ix.hdr[2 * s] = make_uint4(0u - 2u, empty.o_tot - 4u, empty.o_ea - 4u, empty.o_es - 4u);
            ix.hdr[2 * s + 1] = make_uint4(1u | kHdrPark | kHdrTrunc, 0u, 0u, 0u);
            atomicAdd(&ix.ctrl[4], 1u);
        }
        return;
    }
    const bool active = lane < K;
    int32_t pa = 0, ps = 0;
    for (int32_t j = 0; j < K; ++j) {
        const int32_t aj = __builtin_amdgcn_readlane(st_acc, j);
        const uint32_t tj = (uint32_t)__builtin_amdgcn_readlane((int)st_tot, j);
        pa += (aj > st_acc || (aj == st_acc && j < lane)) ? 1 : 0;
        ps += (tj < st_tot || (tj == st_tot && j < lane)) ? 1 : 0;
    }
    uint8_t *body = ix.pool + off;
    if (active) {
        ((uint16_t *)body)[pa] = (uint16_t)(st_acc - lo + 1);
        ((uint32_t *)(body + lay.o_tot))[ps] = st_tot;
        body[lay.o_ra + pa] = (uint8_t)lane;
        body[lay.o_rs + ps] = (uint8_t)lane;
        ix.step_row[rec + lane] = tv.orig_r[(int64_t)b * tv.Vp + seg + st_pos];
    }
    if (lane == 0) {
        ((uint16_t *)body)[K] = 0;
        ((uint32_t *)(body + lay.o_tot))[K] = 0xFFFFFFFFu;
    }
    uint32_t *ea = (uint32_t *)(body + lay.o_ea), *es = (uint32_t *)(body + lay.o_es);
    for (int32_t j = 1; j <= (K >> 1); ++j) {
        const uint64_t ma = __ballot(active && pa < 2 * j);
        const uint64_t ms = __ballot(active && ps < 2 * j);
        if (lane == 0) {
            if (wide) {
                ea[2 * (j - 1)] = (uint32_t)ma; ea[2 * (j - 1) + 1] = (uint32_t)(ma >> 32);
                es[2 * (j - 1)] = (uint32_t)ms; es[2 * (j - 1) + 1] = (uint32_t)(ms >> 32);
            } else {
                ea[j - 1] = (uint32_t)ma;
                es[j - 1] = (uint32_t)ms;
            }
        }
    }
    if (lane == 0) {
        const uint32_t esz = wide ? 8u : 4u;
        ix.hdr[2 * s] = make_uint4(off - 2u, off + lay.o_tot - 4u, off + lay.o_ea - esz, off + lay.o_es - esz);
        ix.hdr[2 * s + 1] = make_uint4((uint32_t)(K + 1) | (wide ? kHdrWide : 0u) | (trunc ? kHdrTrunc : 0u) | kHdrIndexed,
                                       (uint32_t)lo, rec, off + lay.size);
        atomicMax(&ix.ctrl[2], (uint32_t)K);
        if (trunc) atomicAdd(&ix.ctrl[3], 1u);
        atomicAdd(&ix.ctrl[5], (uint32_t)K);
    }
}

// ---------------------------------------------------------------- lookup

#define INFAAS_LDS __attribute__((address_space(3)))

// Readers of index memory by 32-bit byte address: an LDS address, or an offset from a global base.
struct LdsMem {
    __device__ __forceinline__ uint32_t ld32(uint32_t a) const { return *(const INFAAS_LDS uint32_t *)a; }
    __device__ __forceinline__ uint32_t ld16(uint32_t a) const { return *(const INFAAS_LDS uint16_t *)a; }
    __device__ __forceinline__ uint32_t ld8(uint32_t a) const { return *(const INFAAS_LDS uint8_t *)a; }
    __device__ __forceinline__ v4u ld128(uint32_t a) const { return *(const INFAAS_LDS v4u *)a; }
};
struct GlobalMem {
    const uint8_t *p;
    __device__ __forceinline__ uint32_t ld32(uint32_t a) const { return *(const uint32_t *)(p + a); }
    __device__ __forceinline__ uint32_t ld16(uint32_t a) const { return *(const uint16_t *)(p + a); }
    __device__ __forceinline__ uint32_t ld8(uint32_t a) const { return p[a]; }
    __device__ __forceinline__ v4u ld128(uint32_t a) const { return *(const v4u *)(p + a); }
};

// kN queries of one lane against the index, interleaved so that their dependent reads overlap.
// Branch-free apart from wave-uniform conditions; every read stays inside a body plus its slack
// (slices that cannot be used point at the empty dummy body).
//   bodies : memory that the header's addresses refer to
//   hdrs   : memory holding the slice headers, hdr0 = address of header 0
//   nit    : binary-search iterations that cover the largest K of the whole index
// Header of a slice: h0 = {acc keys - 2, tot keys - 4, ea - one entry, es - one entry},
//                    h1 = {K + 1 | flags, acc base, first entry in step_row, body end}.
// Outputs ans (row or -1) and park (query must be finished by the slow path).
template <int kN, class Mem, class HMem>
__device__ __forceinline__ void decide_n(const TableView &tv, const int32_t *__restrict__ step_row,
                                         const Mem &bodies, const HMem &hdrs, uint32_t hdr0, int nit,
                                         const int32_t (&task)[kN], const int32_t (&slo)[kN],
                                         const int32_t (&min_acc)[kN], const int32_t (&bidx)[kN],
                                         int32_t (&ans)[kN], bool (&park)[kN])
{
    bool valid[kN];
    v4u h0[kN], h1[kN];
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        valid[k] = (uint32_t)task[k] < (uint32_t)tv.T && (uint32_t)bidx[k] < (uint32_t)tv.B && slo[k] >= 0;
        const uint32_t s = valid[k] ? (uint32_t)(task[k] * tv.B + bidx[k]) : 0u;
        h0[k] = hdrs.ld128(hdr0 + s * kHdrBytes);
        h1[k] = hdrs.ld128(hdr0 + s * kHdrBytes + 16);
    }
    // binary searches on byte addresses: key number j (1-based) of a slice sits at keys + j * size
    uint32_t dd[kN], pa[kN], la[kN], pt[kN], lt[kN];
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const uint32_t k1 = h1[k].x & 0xFFu;
        const int32_t base = (int32_t)h1[k].y;
        uint32_t d = (uint32_t)min_acc[k] - (uint32_t)base;
        d = d < 65535u ? d : 65535u;
        dd[k] = min_acc[k] > base ? d + 1u : 1u;
        pa[k] = h0[k].x;
        la[k] = h0[k].x + 2u * k1;
        pt[k] = h0[k].y;
        lt[k] = h0[k].y + 4u * k1;
    }
#pragma unroll
    for (int it = 5; it >= 0; --it) {
        if (it < nit) {
#pragma unroll
            for (int k = 0; k < kN; ++k) {
                const uint32_t ca = pa[k] + (2u << it), ct = pt[k] + (4u << it);
                const uint32_t ka = bodies.ld16(ca < la[k] ? ca : la[k]);
                const uint32_t kt = bodies.ld32(ct < lt[k] ? ct : lt[k]);
                pa[k] = ka >= dd[k] ? ca : pa[k];
                pt[k] = kt <= (uint32_t)slo[k] ? ct : pt[k];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        const bool wide = (h1[k].x & kHdrWide) != 0;
        const uint32_t sh = wide ? 3u : 2u;
        const uint32_t p = (pa[k] - h0[k].x) >> 1, ps = (pt[k] - h0[k].y) >> 2;
        const uint32_t a_ra = lt[k] + 3u;                       // ra[-1]
        const uint32_t a_rs = a_ra + (((h1[k].x & 0xFFu) + 2u) & ~3u);
        const uint32_t ja = p >> 1, js = ps >> 1;
        const uint32_t ea = h0[k].z + (ja << sh), es = h0[k].w + (js << sh);
        uint32_t a_lo = bodies.ld32(ea), a_hi = bodies.ld32(ea + 4);
        uint32_t s_lo = bodies.ld32(es), s_hi = bodies.ld32(es + 4);
        const uint32_t ra = bodies.ld8(a_ra + p);
        const uint32_t rs = bodies.ld8(a_rs + ps);
        a_lo = ja ? a_lo : 0u;
        a_hi = (ja && wide) ? a_hi : 0u;
        s_lo = js ? s_lo : 0u;
        s_hi = (js && wide) ? s_hi : 0u;
        const uint64_t A = ((uint64_t)a_hi << 32 | a_lo) | ((uint64_t)(p & 1u) << ra);
        const uint64_t Sm = ((uint64_t)s_hi << 32 | s_lo) | ((uint64_t)(ps & 1u) << rs);
        const uint64_t m = A & Sm;
        const bool hit = valid[k] && m != 0ull;
        const uint32_t step = hit ? h1[k].z + (uint32_t)__builtin_ctzll(m | (1ull << 63)) : 0u;
        const int32_t row = step_row[step];
        ans[k] = hit ? row : -1;
        park[k] = valid[k] && ((h1[k].x & kHdrPark) || (!hit && (h1[k].x & kHdrTrunc)));
    }
}

template <bool kLds>
__global__ __launch_bounds__(kSelThreads) void k_index_select(TableView tv, IndexView ix, QueryView q,
                                                              int32_t *__restrict__ defer_q,
                                                              uint32_t lds_cap, int32_t per_block_cap)
{
    extern __shared__ __align__(16) uint32_t lds_w[];  // [16 B control][S headers][lds_cap bytes of bodies]
    uint32_t &s_defer = lds_w[0];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t hdr_bytes = kLds ? (uint32_t)tv.S * kHdrBytes : 0u;
    const uint32_t lds_hdr0 = (uint32_t)(uintptr_t)(INFAAS_LDS uint32_t *)lds_w + kLdsCtrlBytes;  // LDS address of header 0
    if (kLds) {
        // headers: rebased onto the LDS copy; slices whose body is not resident are parked
        for (uint32_t s = tid; s < (uint32_t)tv.S; s += kSelThreads) {
            uint4 g0 = ix.hdr[2 * s], g1 = ix.hdr[2 * s + 1];
            const bool resident = !(g1.x & kHdrPark) && g1.w <= lds_cap;
            if (!resident) {
                const BodyLayout e(0, false);
                g0 = make_uint4(0u - 2u, e.o_tot - 4u, e.o_ea - 4u, e.o_es - 4u);
                g1 = make_uint4(1u | kHdrPark, 0u, 0u, 0u);
            }
            const uint32_t rebase = lds_hdr0 + hdr_bytes;   // LDS address of pool offset 0
            g0.x += rebase; g0.y += rebase; g0.z += rebase; g0.w += rebase;
            *(uint4 *)(lds_w + (kLdsCtrlBytes / 4) + s * (kHdrBytes / 4)) = g0;
            *(uint4 *)(lds_w + (kLdsCtrlBytes / 4) + s * (kHdrBytes / 4) + 4) = g1;
        }
        uint32_t used = ix.ctrl[0];
        used = used < lds_cap ? used : lds_cap;
        const uint32_t *gp = (const uint32_t *)ix.pool;
        for (uint32_t i = tid; i < (used >> 2); i += kSelThreads)
            lds_w[((kLdsCtrlBytes + hdr_bytes) >> 2) + i] = gp[i];
    }
    if (tid == 0) s_defer = 0;
    __syncthreads();

    const uint32_t max_k = ix.ctrl[2];
    const int nit = 32 - __builtin_clz(max_k | 1u);
    const LdsMem lmem{};
    const GlobalMem gbody{ix.pool};
    const GlobalMem ghdr{(const uint8_t *)ix.hdr};
    int32_t *region = defer_q + (int64_t)blockIdx.x * per_block_cap;

    const bool aligned = ((((uintptr_t)q.task) | ((uintptr_t)q.slo) | ((uintptr_t)q.min_acc) |
                           ((uintptr_t)q.bidx) | ((uintptr_t)q.out)) & 15u) == 0;
    const int32_t ntiles = (q.n + kIndexTile - 1) / kIndexTile;
    for (int32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int32_t i0 = tile * kIndexTile + tid * kPerThread;
        int32_t tk[kPerThread], sl[kPerThread], am[kPerThread], bi[kPerThread];
        const bool vec = aligned && i0 + kPerThread <= q.n;
        if (vec) {
            const v4i a = __builtin_nontemporal_load((const v4i *)(q.task + i0));
            const v4i b = __builtin_nontemporal_load((const v4i *)(q.slo + i0));
            const v4i c = __builtin_nontemporal_load((const v4i *)(q.min_acc + i0));
            const v4i d = __builtin_nontemporal_load((const v4i *)(q.bidx + i0));
            tk[0] = a.x; tk[1] = a.y; tk[2] = a.z; tk[3] = a.w;
            sl[0] = b.x; sl[1] = b.y; sl[2] = b.z; sl[3] = b.w;
            am[0] = c.x; am[1] = c.y; am[2] = c.z; am[3] = c.w;
            bi[0] = d.x; bi[1] = d.y; bi[2] = d.z; bi[3] = d.w;
        } else {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {
                const bool in = i0 + k < q.n;
                tk[k] = in ? q.task[i0 + k] : -1;   // -1: invalid task, decided as "nothing feasible"
                sl[k] = in ? q.slo[i0 + k] : 0;
                am[k] = in ? q.min_acc[i0 + k] : 0;
                bi[k] = in ? q.bidx[i0 + k] : 0;
            }
        }
        int32_t ans[kPerThread];
        bool df[kPerThread];
        if (kLds) decide_n<kPerThread>(tv, ix.step_row, lmem, lmem, lds_hdr0, nit, tk, sl, am, bi, ans, df);
        else decide_n<kPerThread>(tv, ix.step_row, gbody, ghdr, 0u, nit, tk, sl, am, bi, ans, df);
        if (vec) {
            const v4i r = {ans[0], ans[1], ans[2], ans[3]};
            __builtin_nontemporal_store(r, (v4i *)(q.out + i0));
        } else {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k)
                if (i0 + k < q.n) q.out[i0 + k] = ans[k];
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const uint64_t mask = __ballot(df[k]);
            if (mask) {
                const int leader = (int)__builtin_ctzll(mask);
                uint32_t base = 0;
                if (lane == leader) base = atomicAdd(&s_defer, (uint32_t)__builtin_popcountll(mask));
                base = (uint32_t)__builtin_amdgcn_readlane((int)base, leader);
                if (df[k]) region[base + lanes_below(mask)] = i0 + k;
            }
        }
    }

    // ---- parked queries: index copy in global memory, then the rank-ordered scan
    __syncthreads();
    const uint32_t nd = s_defer;
    for (uint32_t j0 = wave * 64; j0 < nd; j0 += kSelThreads) {
        const uint32_t j = j0 + lane;
        const bool have = j < nd;
        const int32_t qi = have ? __hip_atomic_load(&region[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        const int32_t task[1] = {have ? q.task[qi] : -1};
        const int32_t slo[1] = {q.slo[qi]}, min_acc[1] = {q.min_acc[qi]}, bidx[1] = {q.bidx[qi]};
        int32_t ans[1];
        bool pk[1];
        decide_n<1>(tv, ix.step_row, gbody, ghdr, 0u, nit, task, slo, min_acc, bidx, ans, pk);
        uint64_t todo = __ballot(have && pk[0]);
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int32_t t = __builtin_amdgcn_readlane(task[0], l), b = __builtin_amdgcn_readlane(bidx[0], l);
            const int32_t am = __builtin_amdgcn_readlane(min_acc[0], l);
            const uint32_t lim = (uint32_t)__builtin_amdgcn_readlane(slo[0], l);
            const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
            const int64_t col = (int64_t)b * tv.Vp + seg;
            int32_t found = -1;
            for (int32_t blk = 0; blk < L; blk += 64) {
                const int32_t pos = blk + lane;
                const bool ok = pos < L && tv.acc_r[col + pos] >= am && tv.tot_r[col + pos] <= lim;
                const uint64_t bm = __ballot(ok);
                if (bm) { found = blk + (int32_t)__builtin_ctzll(bm); break; }
            }
            if (lane == l) ans[0] = found >= 0 ? tv.orig_r[col + found] : -1;
        }
        if (have) q.out[qi] = ans[0];
    }
}

}  // namespace

// ---------------------------------------------------------------- launchers

hipError_t launch_index_build(const TableView &tv, const IndexView &ix, hipStream_t st)
{
    if (tv.S <= 0) return hipSuccess;
    k_index_build<<<tv.S, 64, 0, st>>>(tv, ix);
    return hipGetLastError();
}

int index_select_blocks(int num_cus) { return num_cus; }

hipError_t launch_index_select(const TableView &tv, const IndexView &ix, const QueryView &q,
                               int32_t *defer_q, uint32_t lds_bytes, int num_cus, hipStream_t st)
{
    const int blocks = index_select_blocks(num_cus);
    const int32_t ntiles = (q.n + kIndexTile - 1) / kIndexTile;
    const int32_t per_block_cap = ((ntiles + blocks - 1) / blocks) * kIndexTile;
    if (lds_bytes > 0) {
        const uint32_t hdr_bytes = (uint32_t)tv.S * kHdrBytes;
        hipError_t e = hipFuncSetAttribute((const void *)k_index_select<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        k_index_select<true><<<blocks, kSelThreads, lds_bytes, st>>>(tv, ix, q, defer_q,
                                                                    lds_bytes - hdr_bytes - kLdsCtrlBytes, per_block_cap);
    } else {
        k_index_select<false><<<blocks, kSelThreads, kLdsCtrlBytes, st>>>(tv, ix, q, defer_q, 0u, per_block_cap);
    }
    return hipGetLastError();
}

}  // namespace infaas
