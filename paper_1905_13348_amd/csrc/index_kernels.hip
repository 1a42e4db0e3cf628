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
    if (L == 0) {  // no variants: the K = 0 dummy body answers "nothing feasible"
        if (lane == 0) ix.hdr[s] = make_uint4(0u, kHdrIndexed, 0u, 0u);
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
            ix.hdr[s] = make_uint4(0u, kHdrTrunc, 0u, 0u);
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
        ix.hdr[s] = make_uint4(off, (uint32_t)K | (wide ? kHdrWide : 0u) | (trunc ? kHdrTrunc : 0u) | kHdrIndexed,
                               (uint32_t)lo, rec);
        atomicMax(&ix.ctrl[2], (uint32_t)K);
        if (trunc) atomicAdd(&ix.ctrl[3], 1u);
        atomicAdd(&ix.ctrl[5], (uint32_t)K);
    }
}

// ---------------------------------------------------------------- lookup

struct LdsMem {
    const uint32_t *w;
    __device__ __forceinline__ uint32_t ld32(uint32_t off) const { return w[off >> 2]; }
    __device__ __forceinline__ uint32_t ld16(uint32_t off) const { return ((const uint16_t *)w)[off >> 1]; }
    __device__ __forceinline__ uint32_t ld8(uint32_t off) const { return ((const uint8_t *)w)[off]; }
};
struct GlobalMem {
    const uint8_t *p;
    __device__ __forceinline__ uint32_t ld32(uint32_t off) const { return *(const uint32_t *)(p + off); }
    __device__ __forceinline__ uint32_t ld16(uint32_t off) const { return *(const uint16_t *)(p + off); }
    __device__ __forceinline__ uint32_t ld8(uint32_t off) const { return p[off]; }
};

// Bit set of the steps that satisfy (min_acc, slo) in the body at byte offset `body`.
// Branch-free; every read stays inside the body plus its slack.  `nit` = search iterations,
// enough for the largest K of the whole index.
template <class Mem>
__device__ __forceinline__ uint64_t lookup_mask(const Mem &mem, uint32_t body, uint32_t K,
                                                bool wide, int32_t base, int32_t min_acc,
                                                uint32_t slo, int nit)
{
    const BodyLayout lay(K, wide);
    const uint32_t k1 = K + 1;
    // accuracy: keys are acc - base + 1 (>= 1), descending; count those >= dd
    uint32_t dd = (uint32_t)min_acc - (uint32_t)base;
    dd = dd < 65535u ? dd : 65535u;
    dd = min_acc > base ? dd + 1u : 1u;
    uint32_t p = 0, ps = 0;
    for (int it = nit - 1; it >= 0; --it) {
        const uint32_t st = 1u << it;
        uint32_t pr = p + st, qr = ps + st;
        uint32_t ia = pr < k1 ? pr : k1, is = qr < k1 ? qr : k1;
        const uint32_t ka = mem.ld16(body + 2 * ia - 2);
        const uint32_t ks = mem.ld32(body + lay.o_tot + 4 * is - 4);
        p = ka >= dd ? pr : p;
        ps = ks <= slo ? qr : ps;
    }
    // bit sets: even counts are stored, odd counts add the bit of the next step
    const uint32_t ja = p >> 1, js = ps >> 1;
    const uint32_t ea_i = ja ? ja - 1 : 0, es_i = js ? js - 1 : 0;
    uint64_t A, Sm;
    if (wide) {
        A = (uint64_t)mem.ld32(body + lay.o_ea + 8 * ea_i) | ((uint64_t)mem.ld32(body + lay.o_ea + 8 * ea_i + 4) << 32);
        Sm = (uint64_t)mem.ld32(body + lay.o_es + 8 * es_i) | ((uint64_t)mem.ld32(body + lay.o_es + 8 * es_i + 4) << 32);
    } else {
        A = mem.ld32(body + lay.o_ea + 4 * ea_i);
        Sm = mem.ld32(body + lay.o_es + 4 * es_i);
    }
    A = ja ? A : 0ull;
    Sm = js ? Sm : 0ull;
    const uint32_t ra = mem.ld8(body + lay.o_ra + (p ? p - 1 : 0));
    const uint32_t rs = mem.ld8(body + lay.o_rs + (ps ? ps - 1 : 0));
    A |= (p & 1u) ? (1ull << ra) : 0ull;
    Sm |= (ps & 1u) ? (1ull << rs) : 0ull;
    return A & Sm;
}

struct Decision {
    int32_t ans;
    bool defer;
};

// One query against the index held in `mem` (header array `hdr`).  kLds: bodies beyond
// lds_cap bytes are not resident and the query is parked.
template <bool kLds, class Mem, class HdrPtr>
__device__ __forceinline__ Decision decide(const TableView &tv, const IndexView &ix, const Mem &mem,
                                           HdrPtr hdr, uint32_t lds_cap, int nit, int32_t task,
                                           int32_t slo, int32_t min_acc, int32_t bidx)
{
    const bool valid = (uint32_t)task < (uint32_t)tv.T && (uint32_t)bidx < (uint32_t)tv.B && slo >= 0;
    const uint32_t s = valid ? (uint32_t)(task * tv.B + bidx) : 0u;
    const uint4 h = hdr[s];
    uint32_t K = h.y & 0xFFu;
    const bool wide = (h.y & kHdrWide) != 0;
    bool usable = valid && (h.y & kHdrIndexed);
    if (kLds) usable = usable && (h.x + BodyLayout(K, wide).size <= lds_cap);
    K = usable ? K : 0u;
    const uint32_t body = usable ? h.x : 0u;
    const uint64_t m = lookup_mask(mem, body, K, usable && wide, (int32_t)h.z, min_acc, (uint32_t)slo, nit);
    const bool hit = m != 0ull;
    const uint32_t step = hit ? (usable ? h.w : 0u) + (uint32_t)__builtin_ctzll(m | (1ull << 63)) : 0u;
    const int32_t row = ix.step_row[step];
    Decision d;
    d.ans = hit ? row : -1;
    d.defer = valid && (!usable || (!hit && (h.y & kHdrTrunc)));
    return d;
}

template <bool kLds>
__global__ __launch_bounds__(kSelThreads) void k_index_select(TableView tv, IndexView ix, QueryView q,
                                                              int32_t *__restrict__ defer_q,
                                                              uint32_t lds_cap, int32_t per_block_cap)
{
    extern __shared__ __align__(16) uint32_t lds_w[];  // [S * 4 header words][lds_cap bytes of bodies]
    __shared__ uint32_t s_defer;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t hdr_words = kLds ? (uint32_t)tv.S * 4u : 0u;
    if (kLds) {
        const uint32_t *gh = (const uint32_t *)ix.hdr;
        for (uint32_t i = tid; i < hdr_words; i += kSelThreads) lds_w[i] = gh[i];
        uint32_t used = ix.ctrl[0];
        used = used < lds_cap ? used : lds_cap;
        const uint32_t *gp = (const uint32_t *)ix.pool;
        for (uint32_t i = tid; i < (used >> 2); i += kSelThreads) lds_w[hdr_words + i] = gp[i];
    }
    if (tid == 0) s_defer = 0;
    __syncthreads();

    const uint32_t max_k = ix.ctrl[2];
    const int nit = 32 - __builtin_clz(max_k | 1u);
    const LdsMem lmem{lds_w + hdr_words};
    const GlobalMem gmem{ix.pool};
    const uint4 *lhdr = (const uint4 *)lds_w;
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
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            Decision d = kLds ? decide<true>(tv, ix, lmem, lhdr, lds_cap, nit, tk[k], sl[k], am[k], bi[k])
                              : decide<false>(tv, ix, gmem, (const uint4 *)ix.hdr, 0u, nit, tk[k], sl[k], am[k], bi[k]);
            ans[k] = d.ans;
            df[k] = d.defer;
        }
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
                uint32_t base = 0;
                if (lane == (int)__builtin_ctzll(mask)) base = atomicAdd(&s_defer, (uint32_t)__builtin_popcountll(mask));
                base = (uint32_t)__builtin_amdgcn_readlane((int)base, (int)__builtin_ctzll(mask));
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
        const int32_t task = have ? q.task[qi] : -1;
        const int32_t slo = q.slo[qi], min_acc = q.min_acc[qi], bidx = q.bidx[qi];
        Decision d = decide<false>(tv, ix, gmem, (const uint4 *)ix.hdr, 0u, nit, task, slo, min_acc, bidx);
        int32_t ans = d.ans;
        uint64_t todo = __ballot(have && d.defer);
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int32_t t = __builtin_amdgcn_readlane(task, l), b = __builtin_amdgcn_readlane(bidx, l);
            const int32_t am = __builtin_amdgcn_readlane(min_acc, l);
            const uint32_t lim = (uint32_t)__builtin_amdgcn_readlane(slo, l);
            const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
            const int64_t col = (int64_t)b * tv.Vp + seg;
            int32_t found = -1;
            for (int32_t blk = 0; blk < L; blk += 64) {
                const int32_t pos = blk + lane;
                const bool ok = pos < L && tv.acc_r[col + pos] >= am && tv.tot_r[col + pos] <= lim;
                const uint64_t bm = __ballot(ok);
                if (bm) { found = blk + (int32_t)__builtin_ctzll(bm); break; }
            }
            if (lane == l) ans = found >= 0 ? tv.orig_r[col + found] : -1;
        }
        if (have) q.out[qi] = ans;
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
        const uint32_t hdr_bytes = (uint32_t)tv.S * 16u;
        hipError_t e = hipFuncSetAttribute((const void *)k_index_select<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        k_index_select<true><<<blocks, kSelThreads, lds_bytes, st>>>(tv, ix, q, defer_q,
                                                                    lds_bytes - hdr_bytes, per_block_cap);
    } else {
        k_index_select<false><<<blocks, kSelThreads, 0, st>>>(tv, ix, q, defer_q, 0u, per_block_cap);
    }
    return hipGetLastError();
}

}  // namespace infaas
