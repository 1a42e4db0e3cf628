// Staircase index of the variant selection (Section 4.1 of the INFaaS paper): the same
// answers as the exhaustive scan, reached through a per-slice structure that keeps only the
// variants that can ever be chosen.  The paper's own controller answers in milliseconds where
// its brute-force search needs ~100 ms because its metadata store keeps sorted sets
// (Sections 5 and 6.4); this is the exact, batched GPU counterpart of that idea.
//
//   k_index_build  : one wavefront per (task, batch) slice finds the "steps" (variants that no
//                    cheaper one dominates), in rounds over a shrinking list of candidates, then
//                    writes sorted keys and bit sets for them (layout: internal.h)
//   k_index_select : one lane per query.  The whole index is mirrored in LDS; a query costs two
//                    5-probe binary searches in LDS, two bit-set reads, one AND and one count-
//                    trailing-zeros.  Queries the first body of their slice cannot decide (no
//                    fitting step among its first 31, slice not resident, staircase truncated)
//                    are parked in a queue of the wavefront and finished by it, 64 at a time or
//                    when it runs out of work: second body, index copy in global memory, and last
//                    a wavefront-wide scan of the rank-ordered slice that stops at the first
//                    feasible variant.  In its closest-variant mode the kernel also parks the
//                    queries that end without a feasible variant and finds, in the same bodies,
//                    the variant that comes closest to their requirements.
#include "internal.h"
#include "lookup_common.h"

namespace infaas {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kPerThread = 4;   // queries per lane and unit, searched interleaved (8 does not fit in 128 VGPRs)
constexpr uint32_t kParkFinal = 1u << 31;          // in a parked record's slice word: the selection is known to be -1
constexpr int kWaveQueue = 64 + 64 * kPerThread;   // parked queries a wavefront can hold: a full pass plus one unit

// ---------------------------------------------------------------- build

// Orders the LDS traffic of ONE wavefront: what its lanes have written is visible to its other lanes.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}


// Body of steps [g0, g0 + kb), held one per lane (lanes g0..g0+kb-1), in two parts: what can be
// computed before the body's place in the pool is known, and the stores.
struct BodyRegs {
    int32_t pa, ps;     // position of this lane's step in the sorted accuracy / latency keys
    uint32_t ma, ms;    // lane p: A[p] and S[p], the steps among the p most accurate / p fastest
};
// Steps [g0, g0 + kb) of a slice: lane j holds step j in (st_acc, st_tot), and p_acc / p_tot hold all
// steps in LDS.  `ranks` is scratch of the wavefront (2 x 64 words).  Values that all lanes need are
// read from LDS (one address for all lanes), so the loops are plain vector code.
__device__ __forceinline__ BodyRegs body_compute(int g0, int kb, int lane, int32_t st_acc, uint32_t st_tot,
                                                 const int32_t *p_acc, const uint32_t *p_tot, int32_t *ranks)
{
    BodyRegs r{0, 0, 0u, 0u};
    const int g1 = g0 + kb;
    for (int j0 = g0; j0 < g1; j0 += 4) {   // four steps per turn, so that their LDS reads overlap
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u < g1 ? j0 + u : g1 - 1;
            const bool in = j0 + u < g1;
            const int32_t aj = p_acc[j];
            const uint32_t tj = p_tot[j];
            r.pa += (int32_t)(in & ((aj > st_acc) | ((aj == st_acc) & (j < lane))));   // (no short-circuit: no branches)
            r.ps += (int32_t)(in & ((tj < st_tot) | ((tj == st_tot) & (j < lane))));
        }
    }
    wave_sync();   // (an earlier body's ranks have been read)
    ranks[lane] = r.pa;
    ranks[64 + lane] = r.ps;
    wave_sync();
    for (int j0 = g0; j0 < g1; j0 += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u < g1 ? j0 + u : g1 - 1;
            const uint32_t bit = j0 + u < g1 ? 1u << (j - g0) : 0u;
            r.ma |= ranks[j] < lane ? bit : 0u;
            r.ms |= ranks[64 + j] < lane ? bit : 0u;
        }
    }
    return r;
}
__device__ __forceinline__ void body_store(uint8_t *body, int g0, int kb, int lane, int32_t st_acc,
                                           uint32_t st_tot, int32_t acc_base, const BodyRegs &r)
{
    const uint32_t re = body_re((uint32_t)kb);
    uint16_t *k_acc = (uint16_t *)body;
    uint32_t *k_tot = (uint32_t *)(body + 2 * re);
    uint32_t *m_a = (uint32_t *)(body + 6 * re);
    uint32_t *m_s = (uint32_t *)(body + 10 * re);
    if (lane >= g0 && lane < g0 + kb) {
        k_acc[r.pa] = (uint16_t)(st_acc - acc_base + 1);
        k_tot[r.ps] = st_tot;
    }
    if (lane >= kb && lane < (int)re) {  // sentinels behind the keys (any lane will do)
        k_acc[lane] = 0;
        k_tot[lane] = 0xFFFFFFFFu;
    }
    if (lane < (int)re) { m_a[lane] = r.ma; m_s[lane] = r.ms; }   // lanes beyond kb hold the full set
}

constexpr int kBuildWaves = 4;                    // slices (wavefronts) per workgroup

// One wavefront per slice, kBuildWaves slices per workgroup.  An entry of the slice is a step exactly
// when no entry ranked before it has at least its accuracy and at most its latency-plus-queue; that
// relation is transitive, so it is enough to test an entry against the earlier STEPS.  The wavefront
// takes in a chunk of the rank-ordered columns, kBuildPer (32 or 16) entries per lane, in registers.  Then
//   1. (first chunk) the steps among the first 64 entries: the first of them is a step (nothing
//      earlier is left), it retires what it dominates among the 64, the next one left is a step, ...;
//   2. a coarse filter: from the steps known so far, a table over ~32 accuracy buckets of the lowest
//      latency-plus-queue among the steps that are at least as accurate as EVERYTHING in the bucket;
//      an entry at or above its bucket's value is dominated for certain and dropped (one LDS read
//      and a compare per entry; nine entries in ten go here).  The others are compacted into a list
//      of candidates in LDS, in rank order;
//   3. rounds over the list until it is empty: the candidates are tested exactly against the steps
//      they have not been tested against yet (four blocks of 64 at a time, a step's values read
//      from its lane once per group; survivors compacted in place), then the steps among the first
//      64 survivors are found as in 1 and leave the list.
// Steps come out in rank order, so when a slice has more than the index keeps, the ones kept are
// its first ones.  The steps sit one per lane (and in LDS); the same wavefront computes the bodies.
// Room in the pool is taken by ONE 64-bit add per workgroup (with one per slice, every slice waited
// microseconds for its turn at the counter).  The larger chunk is faster for slices of thousands of
// variants; the smaller one takes half the LDS and registers, so that twice as many workgroups run
// at a time when there are thousands of slices.
//
// kShare (few slices of thousands of variants each, where the time is one slice's chain of
// dependent steps): ONE slice per workgroup.  Its first wavefront finds the steps as above; then all
// four share the bodies -- each counts and collects over a quarter of the steps, the parts are put
// together through LDS -- while one of them asks for the room in the pool.
template <int kBuildPer, bool kShare>
__global__ __launch_bounds__(64 * kBuildWaves) void k_index_build(TableView tv, IndexView ix)
{
    constexpr int kBuildChunk = 64 * kBuildPer;   // entries of a slice taken in at a time
    constexpr int kLists = kShare ? 1 : kBuildWaves;   // wavefronts that look for steps
    __shared__ int32_t c_acc_all[kLists][kBuildChunk];    // candidates: accuracy,
    __shared__ uint32_t c_tot_all[kLists][kBuildChunk];   //   latency + queue,
    __shared__ uint16_t c_pos_all[kLists][kBuildChunk];   //   position in the chunk
    __shared__ int32_t p_acc_all[kLists][64];             // steps, in rank order
    __shared__ uint32_t p_tot_all[kLists][64];
    __shared__ int32_t p_pos_all[kLists][64];
    __shared__ uint32_t f_tab_all[kLists][64];            // the coarse filter's table
    __shared__ int32_t ranks_all[kLists][128];            // scratch of body_compute; kShare: the steps' places in their bodies
    __shared__ uint32_t parts[kShare ? kBuildWaves : 1][4][64];   // kShare: what each wavefront found over its quarter of the steps
    __shared__ uint32_t s_size[kBuildWaves], s_steps[kBuildWaves], s_stat[4];
    __shared__ uint32_t s_group[kBuildWaves], s_off[kBuildWaves], s_rec[kBuildWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int mine = kShare ? 0 : wave;                   // the lists this wavefront works on
    int32_t *c_acc = c_acc_all[mine], *p_acc = p_acc_all[mine], *p_pos = p_pos_all[mine];
    uint32_t *c_tot = c_tot_all[mine], *p_tot = p_tot_all[mine], *f_tab = f_tab_all[mine];
    uint16_t *c_pos = c_pos_all[mine];
    const int32_t s = kShare ? (int32_t)blockIdx.x : (int32_t)blockIdx.x * kBuildWaves + wave;
    const bool inside = s < tv.S;
    const int32_t t = inside ? s / tv.B : 0, b = inside ? s - t * tv.B : 0;
    const int32_t seg = tv.seg_off[t], L = inside ? tv.seg_len[t] : 0;
    const int32_t *__restrict__ accc = tv.acc_r + (int64_t)b * tv.Vp + seg;
    const uint32_t *__restrict__ totc = tv.tot_r + (int64_t)b * tv.Vp + seg;

    // ---- phase A: the steps, in rank order; lane j < K holds step j, p_acc / p_tot / p_pos all of them
    int32_t K = 0;
    bool trunc = false;
    int32_t st_acc = 0, st_pos = 0;
    uint32_t st_tot = 0u;
    // Steps among up to 64 candidates held one per lane, lanes [0, nh), in rank order, none of them
    // dominated by a known step.  The new steps are appended to the step registers.
    auto take_head = [&](int32_t nh, int32_t a, uint32_t tt, int32_t pos) {
        bool alive = lane < nh;
        uint64_t rest = __ballot(alive);
        while (rest) {   // candidate l is a step (nothing alive precedes it): retire what it dominates
            const int l = __builtin_ctzll(rest);
            const int32_t al = __builtin_amdgcn_readlane(a, l);
            const uint32_t tl = (uint32_t)__builtin_amdgcn_readlane((int)tt, l);
            alive = alive & !((l < lane) & (al >= a) & (tl <= tt));
            rest = __ballot(alive) & ~((2ull << l) - 1ull);
        }
        const uint64_t ok = __ballot(alive);
        const int32_t k_new = (int32_t)__builtin_popcountll(ok);
        const int32_t at = K + (int32_t)lanes_below(ok);
        if (alive && at < kIndexCap) { p_acc[at] = a; p_tot[at] = tt; p_pos[at] = pos; }
        trunc = K + k_new > kIndexCap;   // more steps than the index keeps: its first ones stay
        K = trunc ? kIndexCap : K + k_new;
        wave_sync();
        st_acc = lane < K ? p_acc[lane] : 0;
        st_tot = lane < K ? p_tot[lane] : 0u;
        st_pos = lane < K ? p_pos[lane] : 0;
    };
    for (int32_t c0 = 0; c0 < L && !trunc && (!kShare || wave == 0); c0 += kBuildChunk) {
        const int32_t n = L - c0 < kBuildChunk ? L - c0 : kBuildChunk;
        int32_t va[kBuildPer];
        uint32_t vt[kBuildPer];
        uint32_t dead = 0u;   // bit k: entry k of this lane is outside the chunk, dominated, or taken care of
#pragma unroll
        for (int k = 0; k < kBuildPer; ++k) {   // unconditional loads (clamped), so that they overlap
            const int32_t i = k * 64 + lane;
            const int32_t j = c0 + (i < n ? i : n - 1);
            va[k] = accc[j];
            vt[k] = totc[j];
            dead |= i >= n ? 1u << k : 0u;
        }
        if (K == 0) {   // 1. nothing is known yet: the first 64 entries, exactly
            take_head(n < 64 ? n : 64, va[0], vt[0], c0 + lane);
            if (trunc) break;
            dead |= 1u;
        }
        // 2. coarse filter.  Accuracies from the lowest (mn) to the highest (mx) of the steps are cut
        // into buckets of 2^sh; table entry 0 is for entries below mn, entry 1 + q for bucket q, entry
        // 33 for entries above mx.
        {
            int32_t mn = p_acc[0], mx = mn;
            for (int j0 = 1; j0 < K; j0 += 8) {   // (eight per turn: the LDS reads overlap)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int32_t aj = p_acc[j0 + u < K ? j0 + u : 0];
                    mn = aj < mn ? aj : mn;
                    mx = aj > mx ? aj : mx;
                }
            }
            const uint32_t range = (uint32_t)mx - (uint32_t)mn;
            const int bits = 32 - __builtin_clz(range | 1u);
            const uint32_t sh = bits > 5 ? (uint32_t)(bits - 5) : 0u;   // range >> sh < 32
            // lane i: the lowest latency-plus-queue among the steps at least as accurate as all of
            // bucket i, i.e. with (accuracy - mn + 1) >> sh >= i (entry 0: every step); none: all ones
            uint32_t f = 0xFFFFFFFFu;
            for (int j0 = 0; j0 < K; j0 += 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = j0 + u < K ? j0 + u : 0;   // (step 0 again: harmless)
                    const uint64_t uj = (uint64_t)((uint32_t)p_acc[j] - (uint32_t)mn) + 1u;
                    const uint32_t tj = p_tot[j];
                    const bool covers = (uint32_t)(uj >> sh) >= (uint32_t)lane;
                    f = (covers & (tj < f)) ? tj : f;
                }
            }
            f_tab[lane] = lane <= 33 ? f : 0xFFFFFFFFu;
            if (lane == 33) f_tab[33] = 0xFFFFFFFFu;   // above every step: never dominated
            wave_sync();
#pragma unroll
            for (int k = 0; k < kBuildPer; ++k) {
                const uint32_t u = (uint32_t)va[k] - (uint32_t)mn;
                uint32_t idx = 1u + (u >> sh);
                idx = idx > 33u ? 33u : idx;
                idx = va[k] < mn ? 0u : idx;
                const uint32_t fv = f_tab[idx];
                dead |= ((fv != 0xFFFFFFFFu) & (fv <= vt[k])) ? 1u << k : 0u;
            }
        }
        // what is left becomes the candidate list, entries [beg, end) of the LDS arrays
        int32_t beg = 0, end = 0;
#pragma unroll
        for (int k = 0; k < kBuildPer; ++k) {
            const bool live = !((dead >> k) & 1u);
            const uint64_t m = __ballot(live);
            const int32_t at = end + (int32_t)lanes_below(m);
            if (live) { c_acc[at] = va[k]; c_tot[at] = vt[k]; c_pos[at] = (uint16_t)(k * 64 + lane); }
            end += (int32_t)__builtin_popcountll(m);
        }
        wave_sync();
        // 3. rounds
        int32_t applied = 0;   // the list has been tested exactly against steps [0, applied)
        while (beg < end) {
            // the candidates against the steps they have not met; survivors compacted in place (four
            // blocks are read before anything is written, and written at or below where they were read)
            int32_t out = beg;
            for (int32_t i0 = beg; i0 < end; i0 += 256) {
                int32_t ca[4];
                uint32_t ct[4];
                uint16_t cp[4];
                bool gone[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int32_t i = i0 + u * 64 + lane;
                    const int32_t ci = i < end ? i : beg;
                    ca[u] = c_acc[ci]; ct[u] = c_tot[ci]; cp[u] = c_pos[ci];
                    gone[u] = i >= end;
                }
                for (int j = applied; j < K; ++j) {
                    const int32_t aj = __builtin_amdgcn_readlane(st_acc, j);
                    const uint32_t tj = (uint32_t)__builtin_amdgcn_readlane((int)st_tot, j);
#pragma unroll
                    for (int u = 0; u < 4; ++u) gone[u] = gone[u] | ((aj >= ca[u]) & (tj <= ct[u]));
                }
                wave_sync();
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint64_t m = __ballot(!gone[u]);
                    if (!gone[u]) {
                        const int32_t to = out + (int32_t)lanes_below(m);
                        c_acc[to] = ca[u]; c_tot[to] = ct[u]; c_pos[to] = cp[u];
                    }
                    out += (int32_t)__builtin_popcountll(m);
                }
            }
            end = out;
            applied = K;
            wave_sync();
            if (beg >= end) break;
            // the steps among the first 64 of them
            const int32_t nh = end - beg < 64 ? end - beg : 64;
            const int32_t hi = beg + (lane < nh ? lane : 0);
            take_head(nh, c_acc[hi], c_tot[hi], c0 + (int32_t)c_pos[hi]);
            if (trunc) break;
            beg += nh;
        }
    }

    if constexpr (kShare) {
        // ---- phase B with one slice per workgroup: the steps are in LDS (p_acc / p_tot / p_pos);
        // wavefront w counts and collects over steps [w q, w q + q), q = K / 4 rounded up
        if (wave == 0 && lane == 0) { s_steps[0] = (uint32_t)K; s_size[0] = trunc ? 1u : 0u; }
        lds_barrier();
        K = (int32_t)s_steps[0];
        trunc = s_size[0] != 0u;
        st_acc = lane < K ? p_acc[lane] : 0;
        st_tot = lane < K ? p_tot[lane] : 0u;
        st_pos = lane < K ? p_pos[lane] : 0;
        const int k0 = K < kBodySteps ? K : kBodySteps, k1 = K - k0;
        const uint32_t r0 = (uint32_t)k0 < ix.hot_rows ? (uint32_t)k0 : ix.hot_rows;
        const uint32_t re0 = body_re(k0), re1 = k1 ? body_re(k1) : 0u;
        const uint32_t rows = (2u * r0 + 3u) & ~3u, size0 = body_bytes(re0);
        const uint32_t size = L > 0 ? rows + size0 + body_bytes(re1) : 0u;   // (a multiple of 4)
        const bool has = L > 0;
        // requested now, used at the end: the caller rows of the steps and the two maxima of the statistics
        const int32_t row = (wave == 0 && lane < K) ? tv.orig_r[(int64_t)b * tv.Vp + seg + st_pos] : 0;
        uint32_t stat_now = 0u;
        if (wave == 0 && lane < 2)
            stat_now = __hip_atomic_load(&ix.ctrl[lane == 0 ? kCtlMaxK0 : kCtlMaxK], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Room in the pool and in step_row.  Without groups the slices are placed in the order of their
        // numbers, so that the layout does not depend on which workgroup was quicker: when the bodies
        // outgrow the LDS mirror of the lookup kernel, the slices it leaves out are always those of the
        // last tasks.  Every slice publishes what it needs; the last wavefront adds up what the slices
        // before its own need, once they have all said so (below).  With groups: one add on the
        // group's counter pair, asked for now by one lane and looked at after the sets.
        const bool grouped = ix.num_groups > 1;
        const unsigned long long add = ((unsigned long long)(uint32_t)K << 32) | size;
        const uint32_t epoch = ix.ctrl[kCtlEpoch];
        if (!grouped && threadIdx.x == 0)
            __hip_atomic_store(ix.slice_room + s, add | ((unsigned long long)epoch << 20), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool asks = grouped && threadIdx.x == 192 && size != 0u;
        const uint32_t grp = grouped ? (uint32_t)ix.task_group[t] : 0u;
        unsigned long long *whole = (unsigned long long *)(ix.ctrl + kCtlPool);
        unsigned long long old = 0;
        if (asks) old = atomicAdd((unsigned long long *)(ix.gctrl + 2 * grp), add);
        const int q = (K + kBuildWaves - 1) / kBuildWaves, j_lo = wave * q, j_hi = j_lo + q < K ? j_lo + q : K;
        const bool second = lane >= k0;   // this lane's step belongs to the second body
        // 1. the place of every step among the keys of its body: how many steps of the body come before it
        uint32_t before = 0;              // by accuracy (low half) and by latency-plus-queue (high half)
        for (int j0 = j_lo; j0 < j_hi; j0 += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u < j_hi ? j0 + u : j_hi - 1;
                const bool in = (j0 + u < j_hi) & ((j >= k0) == second);
                const int32_t aj = p_acc[j];
                const uint32_t tj = p_tot[j];
                before += (uint32_t)(in & ((aj > st_acc) | ((aj == st_acc) & (j < lane))));   // (no short-circuit: no branches)
                before += (uint32_t)(in & ((tj < st_tot) | ((tj == st_tot) & (j < lane)))) << 16;
            }
        }
        parts[wave][0][lane] = before;
        lds_barrier();
        before = parts[0][0][lane] + parts[1][0][lane] + parts[2][0][lane] + parts[3][0][lane];
        const int32_t pa = (int32_t)(before & 0xFFFFu), ps = (int32_t)(before >> 16);
        int32_t *ranks = ranks_all[0];
        if (wave == 0) { ranks[lane] = pa; ranks[64 + lane] = ps; }
        lds_barrier();
        // 2. the sets: lane p collects A[p] and S[p] of both bodies
        uint32_t ma0 = 0u, ms0 = 0u, ma1 = 0u, ms1 = 0u;
        for (int j0 = j_lo; j0 < j_hi; j0 += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u < j_hi ? j0 + u : j_hi - 1;
                const bool in = j0 + u < j_hi, first = j < k0;
                const uint32_t bit = in ? 1u << (first ? j : j - k0) : 0u;
                const bool a_in = ranks[j] < lane, s_in = ranks[64 + j] < lane;
                ma0 |= (first & a_in) ? bit : 0u;
                ms0 |= (first & s_in) ? bit : 0u;
                ma1 |= (!first & a_in) ? bit : 0u;
                ms1 |= (!first & s_in) ? bit : 0u;
            }
        }
        parts[wave][0][lane] = ma0; parts[wave][1][lane] = ms0; parts[wave][2][lane] = ma1; parts[wave][3][lane] = ms1;
        if (asks) {
            uint32_t off = (uint32_t)old, rec = (uint32_t)(old >> 32);
            if (off + size <= ix.region_bytes && rec + (uint32_t)K <= ix.group_step_cap) {
                off += grp * ix.region_bytes; rec += grp * ix.group_step_cap;
            } else {   // the group's region has no room: behind the regions
                const unsigned long long o2 = atomicAdd(whole, add);
                off = (uint32_t)o2; rec = (uint32_t)(o2 >> 32);
            }
            s_off[0] = off; s_rec[0] = rec;
        }
        if (!grouped && wave == 3) {
            // What the slices before this one need, lane by lane.  An entry counts once it carries this
            // build's number.  The wait is bounded: every slice publishes as soon as it knows its steps,
            // whatever the others do, and workgroups start in the order of their numbers; should the
            // entries still not be there after kRoomPolls rounds, the slice goes without a body and
            // its queries are answered by the scan.
            constexpr int kRoomPolls = 1 << 16;
            unsigned long long sum = 0;
            bool got = false;
            for (int poll = 0; poll < kRoomPolls && !got; ++poll) {
                bool ok = true;
                sum = 0;
                for (int32_t i = lane; i < s; i += 64) {
                    const unsigned long long v = __hip_atomic_load(ix.slice_room + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = ok && (((uint32_t)v >> 20) == epoch);
                    sum += v & 0xFFFFFFFF000FFFFFull;
                }
                got = __ballot(!ok) == 0ull;
                if (!got) __builtin_amdgcn_s_sleep(16);
            }
            for (int o = 32; o; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == 0) {
                s_off[0] = got ? ix.ctrl[kCtlPool0] + (uint32_t)sum : 0xFFFFFFFFu;
                s_rec[0] = got ? ix.ctrl[kCtlSteps0] + (uint32_t)(sum >> 32) : 0xFFFFFFFFu;
            }
        }
        if (wave == 2) {   // do the accuracies fit 16-bit keys?
            int32_t hi = __builtin_amdgcn_readfirstlane(st_acc), lo = hi;   // (of lane 0, a step whenever the slice has variants)
            for (int32_t j0 = 1; j0 < K; j0 += 8) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int32_t aj = p_acc[j0 + u < K ? j0 + u : 0];
                    hi = aj > hi ? aj : hi;
                    lo = aj < lo ? aj : lo;
                }
            }
            if (lane == 0) s_group[0] = ((int64_t)hi - (int64_t)tv.acc_base <= 65533 && lo >= tv.acc_base) ? 1u : 0u;
        }
        lds_barrier();   // (also: the room and the verdict on the accuracies are in LDS)
        const uint32_t off = s_off[0], rec = s_rec[0];
        const bool fits = has && (uint64_t)off + size <= ix.pool_bytes && (uint64_t)rec + K <= ix.step_cap && s_group[0] != 0u;
        uint8_t *body0 = ix.pool + off + rows;
        if (!grouped && s == tv.S - 1 && threadIdx.x == 0 && off != 0xFFFFFFFFu) {   // the totals, for the statistics
            ix.ctrl[kCtlPool] = off + size;
            ix.ctrl[kCtlSteps] = rec + (uint32_t)K;
        }
        if (wave <= 1 && fits && (wave == 0 || k1)) {   // wavefront 0 writes the first body, wavefront 1 the second
            const int h = 2 * wave;
            BodyRegs r{pa, ps, parts[0][h][lane] | parts[1][h][lane] | parts[2][h][lane] | parts[3][h][lane],
                       parts[0][h + 1][lane] | parts[1][h + 1][lane] | parts[2][h + 1][lane] | parts[3][h + 1][lane]};
            if (wave == 0) body_store(body0, 0, k0, lane, st_acc, st_tot, tv.acc_base, r);
            else body_store(body0 + size0, k0, k1, lane, st_acc, st_tot, tv.acc_base, r);
        }
        if (wave != 0) return;   // (no barrier follows)
        if (fits && lane < K) {
            ix.step_row[rec + lane] = row;
            if ((uint32_t)lane < r0)   // in reverse in front of the body
                *(uint16_t *)(body0 - 2 - 2 * lane) = (uint16_t)row;
        }
        uint32_t row_hi = 0;   // of the first steps' rows the bits above the low 16 go into the header
        for (uint32_t j = 0; j < r0; ++j)
            row_hi |= ((uint32_t)__builtin_amdgcn_readlane(row, (int)j) >> 16) << (j * ix.row_hi_bits);
        if (lane == 0) {
            if (fits) {
                const uint32_t y = (re0 << kHdrK0Shift) | (re1 << kHdrK1Shift) | (trunc ? kHdrTrunc : 0u) |
                                   ((k1 || trunc) ? kHdrDeep : 0u) | row_hi;
                ix.hdr[s] = make_uint4(off + rows - 4u, y, rec, off + size);
            } else if (has) {   // no body: every query of this slice goes to the rank-ordered scan
                ix.hdr[s] = make_uint4(0u, kEmptyHdrY | kHdrPark | kHdrTrunc | kHdrDeep, 0u, 0u);
            } else {            // no variants: the empty dummy body at offset 0 answers "nothing feasible"
                ix.hdr[s] = make_uint4(0u, kEmptyHdrY, 0u, 4u + body_bytes(2));
            }
        }
        // statistics: lanes 0..3 one word each; the maxima only where they raise what was read above
        if (lane < 4) {
            constexpr int word[4] = {kCtlMaxK0, kCtlMaxK, kCtlTrunc, kCtlNoBody};
            const uint32_t v = lane == 0 ? (fits ? (uint32_t)k0 : 0u) : lane == 1 ? (fits ? (uint32_t)K : 0u)
                             : lane == 2 ? ((fits && trunc) ? 1u : 0u) : ((has && !fits) ? 1u : 0u);
            if (lane >= 2) { if (v) atomicAdd(&ix.ctrl[word[lane]], v); }
            else if (v > stat_now) atomicMax(&ix.ctrl[word[lane]], v);
        }
        return;
    }
    // ---- phase B: one or two bodies of sorted keys and bit sets, computed while the workgroup's
    // request for room in the pool is under way
    const int k0 = K < kBodySteps ? K : kBodySteps, k1 = K - k0;
    const uint32_t r0 = (uint32_t)k0 < ix.hot_rows ? (uint32_t)k0 : ix.hot_rows;
    const uint32_t re0 = body_re(k0), re1 = k1 ? body_re(k1) : 0u;
    const uint32_t rows = (2u * r0 + 3u) & ~3u, size0 = body_bytes(re0);
    const uint32_t size = L > 0 ? rows + size0 + body_bytes(re1) : 0u;   // (a multiple of 4)
    if (lane == 0) {
        s_size[wave] = size; s_steps[wave] = (uint32_t)K;
        s_group[wave] = ix.num_groups > 1 ? (uint32_t)ix.task_group[t] : 0u;
    }
    if (threadIdx.x < 4) s_stat[threadIdx.x] = 0u;
    // caller rows of the steps (requested here, used after the bodies have been computed)
    const int32_t row = lane < K ? tv.orig_r[(int64_t)b * tv.Vp + seg + st_pos] : 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        // room in the pool and in step_row for the slices of the workgroup: one 64-bit add on a pair
        // of counters (bytes in the low word) for every run of slices of one group -- one in all,
        // unless the workgroup straddles two groups.  A slice that its group's region has no room for
        // takes its room behind the regions.
        unsigned long long *whole = (unsigned long long *)(ix.ctrl + kCtlPool);
        for (int w0 = 0; w0 < kBuildWaves;) {
            int w1 = w0;
            uint32_t bytes = 0, steps = 0;
            while (w1 < kBuildWaves && s_group[w1] == s_group[w0]) { bytes += s_size[w1]; steps += s_steps[w1]; ++w1; }
            if (bytes) {
                const uint32_t g = s_group[w0];
                const bool grouped = ix.num_groups > 1;
                unsigned long long *pair = grouped ? (unsigned long long *)(ix.gctrl + 2 * g) : whole;
                const unsigned long long old = atomicAdd(pair, ((unsigned long long)steps << 32) | bytes);
                uint32_t off = (uint32_t)old, rec = (uint32_t)(old >> 32);
                for (int w = w0; w < w1; ++w) {
                    if (!grouped) { s_off[w] = off; s_rec[w] = rec; }
                    else if (off + s_size[w] <= ix.region_bytes && rec + s_steps[w] <= ix.group_step_cap) {
                        s_off[w] = g * ix.region_bytes + off; s_rec[w] = g * ix.group_step_cap + rec;
                    } else if (s_size[w]) {
                        const unsigned long long o2 = atomicAdd(whole, ((unsigned long long)s_steps[w] << 32) | s_size[w]);
                        s_off[w] = (uint32_t)o2; s_rec[w] = (uint32_t)(o2 >> 32);
                    }
                    off += s_size[w]; rec += s_steps[w];
                }
            }
            w0 = w1;
        }
    }
    int32_t hi = st_acc, lo = st_acc;   // (of lane 0, a step whenever the slice has variants)
    hi = __builtin_amdgcn_readfirstlane(hi); lo = hi;
    for (int32_t j0 = 1; j0 < K; j0 += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int32_t aj = p_acc[j0 + u < K ? j0 + u : 0];
            hi = aj > hi ? aj : hi;
            lo = aj < lo ? aj : lo;
        }
    }
    const BodyRegs b0 = body_compute(0, k0, lane, st_acc, st_tot, p_acc, p_tot, ranks_all[wave]);
    BodyRegs b1{0, 0, 0u, 0u};
    if (k1) b1 = body_compute(k0, k1, lane, st_acc, st_tot, p_acc, p_tot, ranks_all[wave]);
    // of the first steps' rows the low 16 bits go in front of the body, the bits above into the header
    uint32_t row_hi = 0;
    for (uint32_t j = 0; j < r0; ++j)
        row_hi |= ((uint32_t)__builtin_amdgcn_readlane(row, (int)j) >> 16) << (j * ix.row_hi_bits);
    __syncthreads();
    const bool has = inside && L > 0;
    const uint32_t off = s_off[wave], rec = s_rec[wave];
    const bool fits = has && (uint64_t)off + size <= ix.pool_bytes && (uint64_t)rec + K <= ix.step_cap &&
                      (int64_t)hi - (int64_t)tv.acc_base <= 65533 && lo >= tv.acc_base;   // 16-bit accuracy keys
    if (fits) {
        uint8_t *body0 = ix.pool + off + rows;
        body_store(body0, 0, k0, lane, st_acc, st_tot, tv.acc_base, b0);
        if (k1) body_store(body0 + size0, k0, k1, lane, st_acc, st_tot, tv.acc_base, b1);
        if (lane < K) {
            ix.step_row[rec + lane] = row;
            if ((uint32_t)lane < r0)   // in reverse in front of the body
                *(uint16_t *)(body0 - 2 - 2 * lane) = (uint16_t)row;
        }
    }
    if (lane == 0 && inside) {
        if (fits) {
            const uint32_t y = (re0 << kHdrK0Shift) | (re1 << kHdrK1Shift) | (trunc ? kHdrTrunc : 0u) |
                               ((k1 || trunc) ? kHdrDeep : 0u) | row_hi;
            ix.hdr[s] = make_uint4(off + rows - 4u, y, rec, off + size);
        } else if (has) {   // no body: every query of this slice goes to the rank-ordered scan
            ix.hdr[s] = make_uint4(0u, kEmptyHdrY | kHdrPark | kHdrTrunc | kHdrDeep, 0u, 0u);
        } else {            // no variants: the empty dummy body at offset 0 answers "nothing feasible"
            ix.hdr[s] = make_uint4(0u, kEmptyHdrY, 0u, 4u + body_bytes(2));
        }
        // statistics, gathered per workgroup first: thousands of slices adding to one word of global
        // memory take their turns at ~10 ns each, and the kernel does not end before the last one
        if (fits) {
            atomicMax(&s_stat[0], (uint32_t)k0);
            atomicMax(&s_stat[1], (uint32_t)K);
            if (trunc) atomicAdd(&s_stat[2], 1u);
        } else if (has) {
            atomicAdd(&s_stat[3], 1u);
        }
    }
    __syncthreads();
    if (threadIdx.x < 4 && s_stat[threadIdx.x]) {
        constexpr int word[4] = {kCtlMaxK0, kCtlMaxK, kCtlTrunc, kCtlNoBody};
        const uint32_t v = s_stat[threadIdx.x];
        uint32_t *g = &ix.ctrl[word[threadIdx.x]];
        if (threadIdx.x >= 2) atomicAdd(g, v);
        else if (v > __hip_atomic_load(g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(g, v);   // (mostly not)
    }
}

// ---------------------------------------------------------------- lookup

// ---- closest variant (the suggestion of Section 4.1 for a query that nothing satisfies): the
// variant of the slice that is first by (requirements missed, latency overshoot, accuracy
// shortfall, rank).  It is always a step.  If some step fits the latency bound it is the most
// accurate of those; else if some step is accurate enough, the fastest of those; else the fastest
// of all, the most accurate among equally fast ones; ties go to the earlier rank throughout.

// Counts of one body: accuracy keys >= dd and latency keys <= lim (none when the bound is negative).
template <class Mem>
__device__ __forceinline__ void body_counts(const Mem &mem, int nit, uint32_t body, uint32_t re, uint32_t dd,
                                            uint32_t lim, bool lim_ok, uint32_t &pa, uint32_t &ps)
{
    const uint32_t la = body + 2u * re, lt = la + 4u * re;
    uint32_t a = body, t = la;
#pragma unroll
    for (int it = 4; it >= 0; --it) {
        if (it < nit) {
            const uint32_t ca = a + (2u << it), ct = t + (4u << it);
            const uint32_t ka = mem.ld16(ca < la ? ca : la, 2u);
            const uint32_t kt = mem.ld32(ct < lt ? ct : lt, 0u);
            a = ka >= dd ? ca : a;
            t = kt <= lim ? ct : t;
        }
    }
    pa = (a - body) >> 1;
    ps = lim_ok ? (t - la) >> 2 : 0u;
}

// Smallest p in 1..re-1 whose set (tbl = address of entry 0 of A or of S, minus 4) meets `mask`.
template <class Mem>
__device__ __forceinline__ uint32_t first_meeting(const Mem &mem, uint32_t tbl, uint32_t re, uint32_t mask)
{
    uint32_t p = 0;   // the largest p found so far whose set misses the mask (set 0 is empty)
#pragma unroll
    for (uint32_t step = 16; step; step >>= 1) {
        const uint32_t c = p + step < re - 1u ? p + step : re - 1u;
        const uint32_t set = mem.ld32(tbl + 4u * c, 4u);
        p = (p + step <= re - 1u && (set & mask) == 0u) ? p + step : p;
    }
    return p + 1u;
}

// What one body offers: the step, and the keys the bodies are compared by.
struct Offer {
    uint32_t tot, acc, step;   // latency-plus-queue key, accuracy key, step number in the body
};
// kind 1: most accurate step among those within the latency bound (ps > 0 of them);
// kind 2: fastest step among those accurate enough (pa > 0 of them);
// kind 3: fastest step of all, the most accurate of equally fast ones.  The body has >= 1 step.
template <class Mem>
__device__ __forceinline__ Offer body_offer(const Mem &mem, int nit, uint32_t body, uint32_t re, int kind,
                                            uint32_t pa, uint32_t ps)
{
    const uint32_t acc_k = body, tot_k = body + 2u * re, a_tbl = body + 6u * re, s_tbl = body + 10u * re;
    Offer o;
    if (kind == 2) {
        const uint32_t mask = mem.ld32(a_tbl + 4u * pa, 4u);
        const uint32_t p = first_meeting(mem, s_tbl, re, mask);
        o.tot = mem.ld32(tot_k + 4u * p, 0u);
        o.acc = 0u;
        o.step = (uint32_t)__builtin_ctz(mem.ld32(s_tbl + 4u * p, 4u) & mask);
        return o;
    }
    uint32_t fast = ps;   // kind 3: the steps that share the smallest latency key
    o.tot = mem.ld32(tot_k + 4u, 0u);
    if (kind == 3) {
        uint32_t unused;
        body_counts(mem, nit, body, re, 0x20000u, o.tot, true, unused, fast);
    }
    const uint32_t mask = mem.ld32(s_tbl + 4u * fast, 4u);
    const uint32_t p = first_meeting(mem, a_tbl, re, mask);
    o.acc = mem.ld16(acc_k + 2u * p, 2u);
    o.step = (uint32_t)__builtin_ctz(mem.ld32(a_tbl + 4u * p, 4u) & mask);
    return o;
}

// Closest step of a slice with one or two bodies (re1 = 0: one): the step number in the slice, or -1
// when the slice has nothing to suggest, and how far that step is from the requirements (from its keys:
// no other memory is read).  body1 follows body0 in memory.  min_acc and acc_base_m1 (= accuracy
// base - 1) turn an accuracy key back into an accuracy.
struct ClosestStep {
    int32_t step;
    HowFar how;
};
// A suggestion and its distance as the 16-byte record the first tier of the complete Case I leaves
// beside every query it lists for the second tier (latency overshoot < 2^33, accuracy shortfall < 2^32).
__device__ __forceinline__ v4i pack_side(int32_t row, const HowFar &h)
{
    return v4i{row, (int32_t)(uint32_t)h.over, (int32_t)(uint32_t)h.shortf,
               h.missed | (int32_t)((h.over >> 32) & 1) << 2 | (int32_t)((h.shortf >> 32) & 1) << 3};
}
__device__ __forceinline__ HowFar unpack_side(const v4i &r)
{
    return HowFar{r.w & 3, (int64_t)(uint32_t)r.y | ((int64_t)((r.w >> 2) & 1) << 32),
                  (int64_t)(uint32_t)r.z | ((int64_t)((r.w >> 3) & 1) << 32)};
}
template <class Mem>
__device__ __forceinline__ ClosestStep closest_step(const Mem &mem, int nit, uint32_t body0, uint32_t re0, uint32_t re1,
                                                    uint32_t dd, int32_t slo, int32_t min_acc, int32_t acc_base_m1)
{
    const ClosestStep none{-1, HowFar{3, 0, 0}};
    if (mem.ld32(body0 + 2u * re0 + 4u, 0u) == 0xFFFFFFFFu) return none;   // first latency key is the sentinel: no steps
    const uint32_t body1 = body0 + body_bytes(re0);
    const bool lim_ok = slo >= 0;
    uint32_t pa0, ps0, pa1 = 0, ps1 = 0;
    body_counts(mem, nit, body0, re0, dd, (uint32_t)slo, lim_ok, pa0, ps0);
    if (re1) body_counts(mem, nit, body1, re1, dd, (uint32_t)slo, lim_ok, pa1, ps1);
    const int kind = (ps0 | ps1) ? 1 : ((pa0 | pa1) ? 2 : 3);
    const bool use0 = kind == 1 ? ps0 > 0 : (kind == 2 ? pa0 > 0 : true);
    const bool use1 = re1 && (kind == 1 ? ps1 > 0 : (kind == 2 ? pa1 > 0 : true));
    Offer o0{0, 0, 0}, o1{0, 0, 0};
    if (use0) o0 = body_offer(mem, nit, body0, re0, kind, pa0, ps0);
    if (use1) o1 = body_offer(mem, nit, body1, re1, kind, pa1, ps1);
    bool second = use1 && !use0;
    if (use0 && use1) {   // ties go to the first body, whose steps rank earlier
        if (kind == 1) second = o1.acc > o0.acc;
        else if (kind == 2) second = o1.tot < o0.tot;
        else second = o1.tot < o0.tot || (o1.tot == o0.tot && o1.acc > o0.acc);
    }
    // A table that serves one state keeps the variants of the other states as entries nothing selects
    // (lowest accuracy key, latency key all ones).  Such an entry can be a step, and it is the closest one
    // exactly when the slice has no variant of the table's state: then there is nothing to suggest.  (Of
    // kind 1 the step is within the latency bound, so it is never such an entry.)
    const Offer o = second ? o1 : o0;
    if (kind != 1 && o.tot == 0xFFFFFFFFu) return none;
    // kind 1: within the latency bound, not accurate enough; 2: accurate enough, too slow; 3: neither
    ClosestStep c;
    c.step = second ? (int32_t)(kBodySteps + o.step) : (int32_t)o.step;
    c.how.missed = kind == 3 ? 2 : 1;
    c.how.over = kind == 1 ? 0 : (int64_t)o.tot - (int64_t)slo;
    c.how.shortf = kind == 2 ? 0 : (int64_t)min_acc - ((int64_t)o.acc + (int64_t)acc_base_m1);
    return c;
}

// kMode 0: selection.  1: selection plus closest-variant suggestion (q.closest).
// 2 and 3: the two tiers of the state-aware selection.  2 is the selection over the first tier's
// table; it also writes q.tier (1 = answered, 0 = not) and lists every valid query it leaves
// unanswered, as a (query, latency bound, accuracy bound, slice) record, in its workgroup's part of
// q.open (q.open_cap records each, as many as the workgroup has queries), the number of records in
// q.open_count[workgroup].  3 takes the records of its workgroup's list instead of the query
// arrays, looks them up in the second tier's table and writes q.out and q.tier (= 2) of those it
// can answer; it must be launched with the same grid as the pass that wrote the lists.
// 4 and 5: as 2 and 3, and the worker that serves each answer goes to q.worker (ix.step_worker for
// answers that are steps of the index, q.row_worker for answers found by the scan).
// 6 and 7: as 2 and 3, and q.closest gets the complete Case I: the selected variant, or for a query
// that neither tier can answer the closest variant of the two tiers (6 writes the first tier's
// suggestion, and how far it is from the requirements, beside every record of its lists (q.open_side);
// 7 compares it with its own).  8 and 9: 6 and 7 with the workers of 4 and 5.
template <bool kLds, int kMode>
__global__ __launch_bounds__(kSelThreads) void k_index_select(TableView tv, IndexView ix, QueryView q,
                                                              int32_t *__restrict__ park_mem, uint32_t lds_cap)
{
    constexpr bool kCase1 = kMode >= 6;
    constexpr bool kClosest = kMode == 1, kFirst = kMode >= 2 && !(kMode & 1);
    constexpr bool kSecond = kMode >= 3 && (kMode & 1);
    constexpr bool kWorker = kMode == 4 || kMode == 5 || kMode == 8 || kMode == 9;
    constexpr bool kSuggest = kClosest || kCase1;   // queries without a feasible variant are parked too, for the suggestion
    extern __shared__ __align__(16) uint32_t lds_w[];  // [16 B control][S + 1 headers][lds_cap bytes of bodies]
    publish_index_stats(tv);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t nhdr = (uint32_t)tv.S + 1u;
    const uint32_t hdr_bytes = kLds ? lds_header_bytes(tv.S) : 0u;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(INFAAS_LDS uint32_t *)lds_w;
    const uint32_t lds_hdr0 = lds_base + kLdsCtrlBytes;
    const uint32_t rebase = lds_hdr0 + hdr_bytes;      // LDS address of pool offset 0
    const bool aligned = ((((uintptr_t)q.task) | ((uintptr_t)q.slo) | ((uintptr_t)q.min_acc) |
                           ((uintptr_t)q.bidx) | ((uintptr_t)q.out) | ((uintptr_t)q.closest) |
                           ((uintptr_t)q.tier) | ((uintptr_t)q.worker)) & 15u) == 0;
    // Work units of one wavefront: 64 lanes x kPerThread consecutive queries.  Unit u belongs to
    // workgroup u mod (number of workgroups): all workgroups move through the query arrays together
    // (measured 5% faster than one contiguous range per workgroup).  Inside a workgroup the
    // wavefronts draw its units from a counter in LDS, because the wavefronts of a SIMD do not
    // advance at the same speed.
    // A lane's queries in a unit: four consecutive ones in every block of 256, so that each 16-byte
    // access of the wavefront covers one contiguous kilobyte.
    constexpr int kUnit = 64 * kPerThread;
    constexpr int kSpan = (kPerThread / 4 - 1) * 256 + 4;           // from a lane's first query to behind its last
    auto qoff = [](int k) -> int32_t { return (k >> 2) * 256 + (k & 3); };   // offset of query k of a lane
    // second tier: the units are blocks of 256 records of the workgroup's own list
    const v4i *open_in = (const v4i *)q.open + (int64_t)blockIdx.x * q.open_cap;
    v4i *open_out = (v4i *)q.open + (int64_t)blockIdx.x * q.open_cap;
    const int32_t open_n = kSecond ? q.open_count[blockIdx.x] : 0;
    if (kSecond && open_n == 0) {   // the whole workgroup: nothing was left open in its share
        if (tid < kLookupStats) ix.stats[blockIdx.x * kLookupStats + tid] = 0u;
        return;
    }
    const int32_t nunits = ((kSecond ? open_n : q.n) + kUnit - 1) / kUnit;
    // Query fields of one unit for this lane (unit < 0: nothing left; the fields then describe a
    // query outside the table).  Second tier: tk holds the slice and bi the query's number (negative: no
    // record).
    struct Fields {
        int32_t unit;   // (first: behind bi, the compiler reads bi[k] and it with one wide load, through memory)
        int32_t tk[kPerThread], sl[kPerThread], am[kPerThread], bi[kPerThread];
    };
    constexpr int32_t kNoRecord = -1;
    auto load_unit = [&](Fields &f, int32_t unit) __attribute__((always_inline)) {
        f.unit = unit;
        const int32_t i0 = unit * kUnit + lane * 4;
        if (unit < 0) {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) { f.tk[k] = kSecond ? tv.S : -1; f.sl[k] = 0; f.am[k] = 0; f.bi[k] = kSecond ? kNoRecord : 0; }
        } else if (kSecond) {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {   // record k of a lane: 64 records behind record k - 1
                const int32_t r = unit * kUnit + k * 64 + lane;
                const v4i e = open_in[r < open_n ? r : 0];
                f.tk[k] = r < open_n ? e.w : tv.S;   // (members in the order of the branch above: the compiler
                f.sl[k] = e.y; f.am[k] = e.z;        // merges the branches' last stores, and through a pointer
                f.bi[k] = r < open_n ? e.x : kNoRecord;   // if they go to different members)
            }
        } else if (aligned && i0 + kSpan <= q.n) {
            // one 32-bit byte offset for all four arrays (n <= 2^28).  Loads and stores are
            // non-temporal: every byte is used once.  (With query arrays that come from HBM, as they
            // do when each call gets a new batch, non-temporal loads were measured 4% faster than
            // ordinary ones and ordinary stores 4% slower; only on arrays that a previous call
            // left in the last-level cache are ordinary loads 1% ahead.)
            const uint32_t off = (uint32_t)i0 * 4u;
#pragma unroll
            for (int h = 0; h < kPerThread / 4; ++h) {
                const v4i a = __builtin_nontemporal_load((const v4i *)((const char *)q.task + off) + 64 * h);
                const v4i b = __builtin_nontemporal_load((const v4i *)((const char *)q.slo + off) + 64 * h);
                const v4i c = __builtin_nontemporal_load((const v4i *)((const char *)q.min_acc + off) + 64 * h);
                const v4i d = __builtin_nontemporal_load((const v4i *)((const char *)q.bidx + off) + 64 * h);
                f.tk[4 * h] = a.x; f.tk[4 * h + 1] = a.y; f.tk[4 * h + 2] = a.z; f.tk[4 * h + 3] = a.w;
                f.sl[4 * h] = b.x; f.sl[4 * h + 1] = b.y; f.sl[4 * h + 2] = b.z; f.sl[4 * h + 3] = b.w;
                f.am[4 * h] = c.x; f.am[4 * h + 1] = c.y; f.am[4 * h + 2] = c.z; f.am[4 * h + 3] = c.w;
                f.bi[4 * h] = d.x; f.bi[4 * h + 1] = d.y; f.bi[4 * h + 2] = d.z; f.bi[4 * h + 3] = d.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {
                const int32_t i = i0 + qoff(k);
                const bool in = i < q.n;
                f.tk[k] = in ? q.task[i] : -1;   // -1: outside the table, answered "nothing feasible"
                f.sl[k] = in ? q.slo[i] : 0;
                f.am[k] = in ? q.min_acc[i] : 0;
                f.bi[k] = in ? q.bidx[i] : 0;
            }
        }
    };

    Fields fa, fb;   // two buffers in rotation: searched now, next
    if (kLds) {
        // Mirror the index: all global loads of a lane (its headers and up to kFillDepth x 16 bytes
        // of bodies) are issued before the first LDS write, so the fill costs about one memory
        // round trip.  The whole LDS capacity is copied, used or not, which keeps the copy
        // independent of any value that would have to be read from memory first.
        // Every workgroup copies the same bytes at the same time; the copy goes in 1 KB chunks, one
        // per wavefront and load, and every wavefront of the device starts at a different chunk, so
        // that the requests spread over all L2 channels.
        constexpr int kFillDepth = 10;
        const uint4 *gp = (const uint4 *)ix.pool;
        uint4 *lp = (uint4 *)(lds_w + ((kLdsCtrlBytes + hdr_bytes) >> 2));
        const uint32_t nvec = (lds_cap < ix.pool_bytes ? lds_cap : ix.pool_bytes) >> 4;
        const uint32_t nchunks = (nvec + 63u) >> 6;
        const uint32_t per_wave = (nchunks + (kSelThreads / 64) - 1) / (kSelThreads / 64);
        const uint32_t start = nchunks ? (blockIdx.x * 11u + (uint32_t)wave * per_wave) % nchunks : 0u;
        uint4 v[kFillDepth];
        uint32_t at[kFillDepth];
        bool ok[kFillDepth];
#pragma unroll
        for (int u = 0; u < kFillDepth; ++u) {
            uint32_t c = start + u;
            c = c >= nchunks ? c - nchunks : c;
            ok[u] = (uint32_t)u < per_wave && (uint32_t)wave * per_wave + u < nchunks && c * 64u + lane < nvec;
            at[u] = ok[u] ? c * 64u + lane : 0u;   // lanes with nothing to copy read vector 0 and drop it
            v[u] = gp[at[u]];                      // unconditional: keeps all loads in flight together
        }
        // headers: rebased onto the LDS copy; slices whose bodies are not resident are parked
        for (uint32_t s = tid; s < nhdr; s += kSelThreads) {
            const uint4 g = ix.hdr[s];
            const bool resident = !(g.y & kHdrPark) && g.w <= lds_cap && g.z < 65536u;
            v2u l;
            l.x = ((resident ? g.x : 0u) + rebase) | (g.y << kLdsAddrBits);   // high row bits above the address
            l.y = resident ? ((g.y & 0xFFFF0000u) | g.z) : (kEmptyHdrY | kHdrPark | kHdrDeep);
            *(v2u *)(lds_w + (kLdsCtrlBytes / 4) + s * (kLdsHdrBytes / 4)) = l;
        }
#pragma unroll
        for (int u = 0; u < kFillDepth; ++u)
            lp[at[u]] = v[u];   // unconditional as well (lanes without work rewrite vector 0 with itself)
        for (uint32_t c0 = kFillDepth; c0 < per_wave; ++c0) {   // only if LDS ever exceeds 160 KB
            uint32_t c = start + c0;
            c = c >= nchunks ? c - nchunks : c;
            const uint32_t i = c * 64u + lane;
            if ((uint32_t)wave * per_wave + c0 < nchunks && i < nvec) lp[i] = gp[i];
        }
    }
    // worker selection: 16-bit workers of the hot steps behind the bodies (lds_cap excludes them)
    const bool hot_w = kLds && kWorker && ix.hot_worker != nullptr;
    const uint32_t hotw_base = rebase + lds_cap;
    if (hot_w) {
        const uint32_t nw = (nhdr - 1u) * ix.hot_rows;   // 16-bit entries; the array has 8 more behind them
        const uint32_t *gw = (const uint32_t *)ix.hot_worker;
        uint32_t *lw = lds_w + ((kLdsCtrlBytes + hdr_bytes + lds_cap) >> 2);
        for (uint32_t i = tid; i < (nw + 1u) >> 1; i += kSelThreads) lw[i] = gw[i];
    }
    if (tid < (int)(kLdsCtrlBytes / 4)) lds_w[tid] = 0u;
    __syncthreads();

    const uint32_t row_hi_mask = (1u << ix.row_hi_bits) - 1u;
    const int32_t acc_base_m1 = tv.acc_base - 1;   // acc_base is above INT32_MIN
    const uint32_t max_k = ix.ctrl[kCtlMaxK0];
    const int nit = 32 - __builtin_clz(max_k | 1u);    // <= 5
    const LdsMem lmem{};
    const GlobalMem gmem{ix.pool};
    // Parked queries of this wavefront: (query, latency bound, accuracy bound, slice) records in a
    // queue of its own in global memory, written and read by this wavefront only.
    v4i *wq = (v4i *)park_mem + ((int64_t)blockIdx.x * (kSelThreads / 64) + wave) * kWaveQueue;
    uint32_t cnt = 0;   // records in the queue (wave-uniform)
    // what became of this wavefront's parked queries (wave-uniform; summed per workgroup at the end)
    uint32_t st_parked = 0, st_second = 0, st_global = 0, st_scanned = 0, st_none = 0;

    uint32_t &s_next = lds_w[2];
    auto next_unit = [&]() -> int32_t {
        uint32_t u = 0;
        if (lane == 0) u = atomicAdd(&s_next, 1u);
        u = (uint32_t)__builtin_amdgcn_readfirstlane((int)u);
        const int64_t unit = kSecond ? (int64_t)u : (int64_t)blockIdx.x + (int64_t)u * gridDim.x;
        return unit < nunits ? (int32_t)unit : -1;
    };
    load_unit(fa, next_unit());
    load_unit(fb, next_unit());
    // Software pipeline.  A wavefront waits for memory once per unit, at the top, where it needs the
    // unit's query fields; that wait also covers everything requested before it.  The rows gathered
    // for a unit are therefore consumed, and its results stored, only after the NEXT unit's wait --
    // one full unit of LDS work after they were requested -- so neither the gather nor the store
    // latency is exposed.  Two buffers of query fields alternate: as soon as a unit has been searched
    // its buffer is refilled with the unit after the next, which leaves that request one full stage
    // to arrive.  (A third buffer, requested a stage earlier, was measured 1% slower.)
    int32_t p_lrow[kPerThread], p_grow[kPerThread], p_i0 = -1;
    uint32_t p_base[kPerThread];
    bool p_inl[kPerThread];
    int32_t p_qi[kPerThread];   // second tier only: where each result goes
    int32_t p_wk[kPerThread];   // worker selection only: the worker of each answer, gathered from global memory ...
    int32_t p_wl[kPerThread];   // ... or its 16-bit copy from LDS (-1: not there)
    auto p_worker = [&](int k) -> int32_t { return p_wl[k] >= 0 ? (p_wl[k] == 0xFFFF ? -1 : p_wl[k]) : p_wk[k]; };
    auto p_val = [&](int k) -> int32_t { return p_inl[k] ? (int32_t)((p_base[k] << 16) | (uint32_t)p_lrow[k]) : p_grow[k]; };
    auto store_unit = [&]() {
        if (p_i0 < 0) return;
        if (kSecond) {   // only the answers: the first tier has written "none" for all of the list
#pragma unroll
            for (int k = 0; k < kPerThread; ++k)
                if (p_qi[k] >= 0 && p_val(k) >= 0) {
                    q.out[p_qi[k]] = p_val(k); q.tier[p_qi[k]] = 2;
                    if (kCase1) q.closest[p_qi[k]] = p_val(k);
                    if (kWorker) q.worker[p_qi[k]] = p_worker(k);
                }
        } else if (aligned && p_i0 + kSpan <= q.n) {
#pragma unroll
            for (int h = 0; h < kPerThread / 4; ++h) {
                const v4i r = {p_val(4 * h), p_val(4 * h + 1), p_val(4 * h + 2), p_val(4 * h + 3)};
                __builtin_nontemporal_store(r, (v4i *)((char *)q.out + (uint32_t)p_i0 * 4u) + 64 * h);
                if (kSuggest) __builtin_nontemporal_store(r, (v4i *)((char *)q.closest + (uint32_t)p_i0 * 4u) + 64 * h);
                if (kFirst) {
                    const v4i t4 = {r.x >= 0, r.y >= 0, r.z >= 0, r.w >= 0};
                    __builtin_nontemporal_store(t4, (v4i *)((char *)q.tier + (uint32_t)p_i0 * 4u) + 64 * h);
                }
                if (kWorker) {
                    const v4i w4 = {p_worker(4 * h), p_worker(4 * h + 1), p_worker(4 * h + 2), p_worker(4 * h + 3)};
                    __builtin_nontemporal_store(w4, (v4i *)((char *)q.worker + (uint32_t)p_i0 * 4u) + 64 * h);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPerThread; ++k)
                if (p_i0 + qoff(k) < q.n) {
                    q.out[p_i0 + qoff(k)] = p_val(k);
                    if (kSuggest) q.closest[p_i0 + qoff(k)] = p_val(k);
                    if (kFirst) q.tier[p_i0 + qoff(k)] = p_val(k) >= 0;
                    if (kWorker) q.worker[p_i0 + qoff(k)] = p_worker(k);
                }
        }
    };
    // One pipeline stage: search the unit in `cur`, then request the unit after the next into it.
    uint32_t &s_open = lds_w[3];   // first tier: records in the workgroup's list so far
    // Room for `count` (wave-uniform, > 0) more records in the workgroup's list: one LDS atomic.
    auto open_room = [&](uint32_t count) -> uint32_t {
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&s_open, count);
        return (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
    };
    auto stage = [&](Fields &cur) __attribute__((always_inline)) {
        const int32_t i0 = kSecond ? 0 : cur.unit * kUnit + lane * 4;
        store_unit();                                   // results of the previous unit
        // slice header; queries outside the table use the header of the empty slice (entry S)
        uint32_t body[kPerThread], y[kPerThread], rec[kPerThread], keys[kPerThread], dd[kPerThread],
            lim[kPerThread], m[kPerThread], sl_of[kPerThread], rbase[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const uint32_t inside = ((uint32_t)cur.tk[k] < (uint32_t)tv.T) & ((uint32_t)cur.bi[k] < (uint32_t)tv.B);
            const uint32_t ok = inside & (uint32_t)(cur.sl[k] >= 0);   // a negative bound admits nothing
            const uint32_t own = __umul24((uint32_t)cur.tk[k], (uint32_t)tv.B) + (uint32_t)cur.bi[k];
            // (a record of the second tier names its slice; one with a negative bound can only get a suggestion)
            const uint32_t s = kSecond ? ((kCase1 && cur.sl[k] < 0) ? (uint32_t)tv.S : (uint32_t)cur.tk[k])
                                       : (ok ? own : (uint32_t)tv.S);
            // the slice a parked record names
            sl_of[k] = kSecond ? (uint32_t)cur.tk[k] : (kSuggest ? (inside ? own : (uint32_t)tv.S) : s);
            if (kLds) {
                const v2u h = lmem.ld64(lds_hdr0 + s * kLdsHdrBytes);
                body[k] = h.x & ((1u << kLdsAddrBits) - 1u); y[k] = h.y; rec[k] = h.y & 0xFFFFu;
                rbase[k] = h.x >> kLdsAddrBits;
            } else {
                const uint4 h = ix.hdr[s];
                body[k] = h.x; y[k] = h.y; rec[k] = h.z;
                rbase[k] = h.y & ((1u << kRowHiField) - 1u);
            }
            keys[k] = (y[k] >> kHdrK0Shift) & 0x3Fu;   // Re of the first body
            dd[k] = acc_threshold(cur.am[k], acc_base_m1);
            lim[k] = (uint32_t)cur.sl[k];
        }
        if (kLds) search_bodies<kPerThread>(lmem, nit, body, keys, dd, lim, m);
        else search_bodies<kPerThread>(gmem, nit, body, keys, dd, lim, m);
        bool df[kPerThread];
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const bool hit = m[k] != 0u;
            const uint32_t step = (uint32_t)__builtin_ctzg(m[k], -1);   // no fitting step: above every count
            // row of the step: from in front of the body (low 16 bits) and the header (the bits above)
            // when it is one of its first hot_rows steps, else from step_row in global memory.  Both
            // reads are issued for every lane (lanes that do not need one read a fixed address) and
            // used after the next wait.  step_row[0] is -1, which is what a lane without a fitting
            // step reads and reports.
            const bool inl = step < ix.hot_rows;
            const uint32_t at = inl ? body[k] - 2u * step : body[k];
            p_lrow[k] = kLds ? (int32_t)lmem.ld16(at, 2u) : (int32_t)gmem.ld16(at, 2u);
            p_base[k] = (rbase[k] >> ((step * ix.row_hi_bits) & 31u)) & row_hi_mask;
            p_grow[k] = *(const int32_t *)((const char *)ix.step_row + ((hit && !inl) ? (rec[k] + step) * 4u : 0u));
            p_inl[k] = inl;
            // the worker of the step: of a hot step from LDS, else by the same kind of gather as the
            // row (entry 0, for no step, is -1)
            if (kWorker) {
                const bool wl = hot_w && inl;
                p_wk[k] = *(const int32_t *)((const char *)ix.step_worker + ((hit && !wl) ? (rec[k] + step) * 4u : 0u));
                p_wl[k] = -1;
                if (hot_w) {   // every lane reads (lanes without a hot step the first entry) and keeps it only if it is its own
                    const uint32_t slice = kSecond ? (uint32_t)cur.tk[k] : sl_of[k];
                    const uint32_t w16 = lmem.ld16(hotw_base + (wl ? (__umul24(slice, ix.hot_rows) + step) * 2u : 0u), 0u);
                    p_wl[k] = wl ? (int32_t)w16 : -1;
                }
            }
            if (kSecond) p_qi[k] = cur.bi[k];
            // parked: a miss that the second body / the scan may still turn into a hit; in the
            // closest-variant mode also every final miss of a query inside the table
            df[k] = !hit && ((int32_t)y[k] < 0 || (kSuggest && sl_of[k] != (uint32_t)tv.S));
            if (kSuggest && (int32_t)y[k] >= 0) sl_of[k] |= kParkFinal;   // nothing feasible: only the suggestion is open
        }
        p_i0 = i0;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            const uint64_t mask = __ballot(df[k]);
            if (mask) {   // parked queries are always inside the table
                // (first word: the query; in the last pass of the complete Case I the record's place in the
                // workgroup's list, where the query and the first tier's suggestion are found)
                if (df[k]) wq[cnt + lanes_below(mask)] = v4i{(kCase1 && kSecond) ? cur.unit * kUnit + k * 64 + lane : kSecond ? cur.bi[k] : i0 + qoff(k),
                                                              cur.sl[k], cur.am[k], (int32_t)sl_of[k]};
                cnt += (uint32_t)__builtin_popcountll(mask);
                st_parked += (uint32_t)__builtin_popcountll(mask);
            }
        }
        if (kFirst) {   // valid queries that end here without an answer go to the second tier
            uint64_t om[kPerThread];
            uint32_t total = 0;
#pragma unroll
            for (int k = 0; k < kPerThread; ++k) {
                om[k] = __ballot(m[k] == 0u && !df[k] && sl_of[k] != (uint32_t)tv.S);
                total += (uint32_t)__builtin_popcountll(om[k]);
            }
            if (total) {
                uint32_t at = open_room(total);
#pragma unroll
                for (int k = 0; k < kPerThread; ++k) {
                    if ((om[k] >> lane) & 1u)
                        open_out[at + lanes_below(om[k])] = v4i{i0 + qoff(k), cur.sl[k], cur.am[k], (int32_t)sl_of[k]};
                    at += (uint32_t)__builtin_popcountll(om[k]);
                }
            }
        }
        load_unit(cur, next_unit());
    };
    // Finishes `count` <= 64 parked queries, records [first, first + count) of the queue.
    auto drain = [&](uint32_t first, uint32_t count) {
        // The records, and the "nothing feasible" stored for these queries by the main loop, must
        // have left this wavefront before they are read back and overwritten.  Writer and reader are
        // the same wavefront, so workgroup scope is enough (a wider release would write back L2).
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        const bool have = (uint32_t)lane < count;
        const int32_t *e = (const int32_t *)(wq + first + (have ? lane : 0));
        int32_t qi = __hip_atomic_load(e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        v4i side{-1, 0, 0, 3};   // last pass of the complete Case I: what the first tier suggests, and how far that is
        if (kCase1 && kSecond) {
            const int32_t r = have ? qi : 0;
            qi = open_in[r].x;
            side = ((const v4i *)q.open_side + (int64_t)blockIdx.x * q.open_cap)[r];
        }
        const int32_t slo = __hip_atomic_load(e + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int32_t min_acc = __hip_atomic_load(e + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int32_t s_ld = __hip_atomic_load(e + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const bool final_miss = kSuggest && have && ((uint32_t)s_ld & kParkFinal);
        const uint32_t s = have ? ((uint32_t)s_ld & ~kParkFinal) : (uint32_t)tv.S;   // idle lanes: the empty slice
        uint32_t y = 0, rec = 0, lbody = rebase, gbody = 0;
        bool resident = false;
        if (kLds) {
            const v2u h = lmem.ld64(lds_hdr0 + s * kLdsHdrBytes);
            resident = !(h.y & kHdrPark);
            lbody = h.x & ((1u << kLdsAddrBits) - 1u); y = h.y; rec = h.y & 0xFFFFu;
        }
        if (__ballot(!resident)) {   // slices without a body in LDS: header from global memory
            const uint4 g = ix.hdr[resident ? (uint32_t)tv.S : s];
            if (!resident) { y = g.y; rec = g.z; gbody = g.x; }
        }
        const bool indexed = !(y & kHdrPark);
        const uint32_t keys0 = (y >> kHdrK0Shift) & 0x3Fu, keys1 = (y >> kHdrK1Shift) & 0x3Fu;   // Re of the bodies
        const uint32_t size0 = body_bytes(keys0);
        const uint32_t dd[1] = {acc_threshold(min_acc, acc_base_m1)}, lim[1] = {(uint32_t)slo};
        int32_t ans = -1, wk = -1;
        auto take_step = [&](uint32_t at) {   // the answer is step `at` of the index
            ans = ix.step_row[at];
            if (kWorker) wk = ix.step_worker[at];
        };
        bool done = final_miss;
        // bodies in global memory (the first one only if the main loop could not use an LDS copy):
        // both are searched together, level by level, so that one body's trips to memory hide the other's
        const bool need_g0 = have && indexed && kLds && !resident && !done;
        const bool need_g1 = have && indexed && keys1 != 0u && !resident && !done;
        if (__ballot(need_g0 | need_g1)) {
            const uint32_t bd[2] = {need_g0 ? gbody : 0u, need_g1 ? gbody + size0 : 0u};
            const uint32_t ks[2] = {need_g0 ? keys0 : 2u, need_g1 ? keys1 : 2u};
            const uint32_t dd2[2] = {dd[0], dd[0]}, lim2[2] = {lim[0], lim[0]};
            uint32_t m[2];
            search_bodies<2>(gmem, nit, bd, ks, dd2, lim2, m);
            const bool hit0 = need_g0 && m[0], hit1 = need_g1 && !hit0 && m[1];
            if (hit0) take_step(rec + __builtin_ctz(m[0]));
            if (hit1) take_step(rec + kBodySteps + __builtin_ctz(m[1]));
            done = done || hit0 || hit1;
            st_global += (uint32_t)__builtin_popcountll(__ballot(hit0));
            st_second += (uint32_t)__builtin_popcountll(__ballot(hit1));
        }
        // second body of a slice whose bodies are in LDS
        const bool need_l1 = have && indexed && keys1 != 0u && resident && !done;
        if (kLds && __ballot(need_l1)) {
            const uint32_t bd[1] = {need_l1 ? lbody + size0 : rebase}, ks[1] = {need_l1 ? keys1 : 2u};
            uint32_t m[1];
            search_bodies<1>(lmem, nit, bd, ks, dd, lim, m);
            if (need_l1 && m[0]) { take_step(rec + kBodySteps + __builtin_ctz(m[0])); done = true; }
            st_second += (uint32_t)__builtin_popcountll(__ballot(need_l1 && m[0]));
        }
        // no body, or both bodies missed and more steps exist: scan the slice in rank order
        uint64_t todo = __ballot(have && !done && (!indexed || (y & kHdrTrunc)));
        if (todo) {
            st_scanned += (uint32_t)__builtin_popcountll(todo);
            const int32_t task = (int32_t)(s / (uint32_t)tv.B), bidx = (int32_t)(s - (uint32_t)task * (uint32_t)tv.B);
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
                if (lane == l) {
                    ans = found >= 0 ? tv.orig_r[col + found] : -1;
                    if (kWorker) wk = found >= 0 ? q.row_worker[ans] : -1;
                }
            }
        }
        st_none += (uint32_t)__builtin_popcountll(__ballot(have && !final_miss && ans < 0));
        if (kSecond) {
            if (have && ans >= 0) {
                q.out[qi] = ans; q.tier[qi] = 2;
                if (kCase1) q.closest[qi] = ans;
                if (kWorker) q.worker[qi] = wk;
            }
        } else if (have && !final_miss) {
            q.out[qi] = ans;
        }
        uint32_t open_at = 0;   // first tier: where this lane's query went in the workgroup's list
        if (kFirst) {   // the main loop has stored tier 0 for a parked query
            if (have && ans >= 0) {
                q.tier[qi] = 1;
                if (kWorker) q.worker[qi] = wk;
            }
            const uint64_t om = __ballot(have && ans < 0);
            if (om) {
                open_at = open_room((uint32_t)__builtin_popcountll(om)) + lanes_below(om);
                if (have && ans < 0) open_out[open_at] = v4i{qi, slo, min_acc, (int32_t)s};
            }
        }
        if (kSuggest) {
            // the suggestion for the queries that ended with nothing feasible
            const bool open = have && ans < 0;
            const bool by_index = open && indexed && !(y & kHdrTrunc);
            int32_t sug = ans;
            HowFar mine{3, 0, 0};   // how far the suggestion is from the requirements
            const bool in_lds = by_index && resident, in_mem = by_index && !resident;
            if (kLds && __ballot(in_lds)) {
                const ClosestStep c = closest_step(lmem, nit, in_lds ? lbody : rebase, in_lds ? keys0 : 2u,
                                                   in_lds ? keys1 : 0u, dd[0], slo, min_acc, acc_base_m1);
                if (in_lds && c.step >= 0) { sug = ix.step_row[rec + (uint32_t)c.step]; mine = c.how; }
            }
            if (__ballot(in_mem)) {
                const ClosestStep c = closest_step(gmem, nit, in_mem ? gbody : 0u, in_mem ? keys0 : 2u,
                                                   in_mem ? keys1 : 0u, dd[0], slo, min_acc, acc_base_m1);
                if (in_mem && c.step >= 0) { sug = ix.step_row[rec + (uint32_t)c.step]; mine = c.how; }
            }
            // slices without a complete index: the whole slice, in rank order, by the wavefront
            uint64_t rest = __ballot(open && !by_index);
            if (rest) {
                const int32_t task = (int32_t)(s / (uint32_t)tv.B), bidx = (int32_t)(s - (uint32_t)task * (uint32_t)tv.B);
                while (rest) {
                    const int l = __builtin_ctzll(rest);
                    rest &= rest - 1;
                    const int32_t t = __builtin_amdgcn_readlane(task, l), b = __builtin_amdgcn_readlane(bidx, l);
                    const int64_t am = __builtin_amdgcn_readlane(min_acc, l), bound = __builtin_amdgcn_readlane(slo, l);
                    HowFar how;
                    const int32_t found = closest_by_scan(tv, t, b, am, bound, lane, &how);
                    if (lane == l) { sug = found; mine = how; }
                }
            }
            if (kCase1 && kFirst && open)   // for the second tier: this tier's suggestion and how far it is
                ((v4i *)q.open_side + (int64_t)blockIdx.x * q.open_cap)[open_at] = pack_side(sug, mine);
            if (kCase1 && kSecond) {
                // the closer of the two tiers' suggestions, by (requirements missed, latency beyond the
                // bound, accuracy below the bound), the first tier's at a tie; q.closest holds the first tier's
                if (open && sug >= 0) {
                    const bool keep_first = side.x >= 0 && closer_or_equal(unpack_side(side), mine);
                    if (!keep_first) q.closest[qi] = sug;
                }
            } else if (have) {
                q.closest[qi] = sug;
            }
        }
    };

    {
        // The rotation is interrupted only when 64 parked queries have collected (one full pass of
        // the wavefront) and resumed where it stopped.
        int phase = 0;
        bool more = true;
        while (more) {
            for (;;) {
                if (phase == 0) {
                    if (fa.unit < 0) { more = false; break; }
                    stage(fa);
                    phase = 1;
                    if (cnt >= 64u) break;
                }
                if (fb.unit < 0) { more = false; break; }
                stage(fb);
                phase = 0;
                if (cnt >= 64u) break;
            }
            store_unit();   // a parked query gets -1 here and its real answer in drain()
            p_i0 = -1;
            while (cnt >= 64u || (!more && cnt > 0u)) {
                const uint32_t c = cnt < 64u ? cnt : 64u;
                drain(cnt - c, c);
                cnt -= c;
            }
        }
    }
    // statistics of this launch, per workgroup (plain stores: nothing waits for them)
    if (lane == 0) {
        const uint32_t st[kLookupStats] = {st_parked, st_second, st_global, st_scanned, st_none};
#pragma unroll
        for (int i = 0; i < kLookupStats; ++i)
            if (st[i]) atomicAdd(&lds_w[4 + i], st[i]);
    }
    __syncthreads();
    if (tid < kLookupStats) ix.stats[blockIdx.x * kLookupStats + tid] = lds_w[4 + tid];
    if (kFirst && tid == 0) q.open_count[blockIdx.x] = (int32_t)s_open;
}

}  // namespace

// ---------------------------------------------------------------- launchers

hipError_t launch_index_build(const TableView &tv, const IndexView &ix, hipStream_t st, const LaunchEvents *ev)
{
    if (tv.S <= 0) return hipSuccess;
    const dim3 block(64 * kBuildWaves);
    // few slices of many variants each: one slice per workgroup, its wavefronts share the bodies
    if (tv.S <= 512 && (int64_t)tv.Vp >= 512 * (int64_t)tv.T)
        return launch_kernel(ev, k_index_build<32, true>, dim3((unsigned)tv.S), block, 0, st, tv, ix);
    const dim3 grid((unsigned)((tv.S + kBuildWaves - 1) / kBuildWaves));
    // up to 1024 slices every workgroup is resident at once whatever its size: the larger chunk
    if (tv.S <= 1024) return launch_kernel(ev, k_index_build<32, false>, grid, block, 0, st, tv, ix);
    return launch_kernel(ev, k_index_build<16, false>, grid, block, 0, st, tv, ix);
}

int index_select_blocks(int num_cus) { return num_cus; }

// Records per workgroup of the lists a first-tier pass over n queries may write: every query of
// the workgroup's share of the units.
int32_t index_open_cap(int32_t n, int num_cus)
{
    const int64_t unit = 64 * kPerThread, blocks = index_select_blocks(num_cus);
    const int64_t nunits = (n + unit - 1) / unit;
    return (int32_t)(((nunits + blocks - 1) / blocks) * unit);
}

size_t index_park_bytes(int num_cus)
{
    return (size_t)index_select_blocks(num_cus) * (kSelThreads / 64) * kWaveQueue * sizeof(v4i);
}

hipError_t launch_index_select(const TableView &tv, const IndexView &ix, const QueryView &q,
                               int32_t *park_mem, uint32_t lds_bytes, int num_cus, hipStream_t st, const LaunchEvents *ev)
{
    const int blocks = index_select_blocks(num_cus);
    if (lds_bytes > 0) {
        const uint32_t fixed = kLdsCtrlBytes + lds_header_bytes(tv.S);
        lds_bytes = fixed + ((lds_bytes - fixed) & ~15u);
        auto kernel = q.pass == 1 ? k_index_select<true, 1> : q.pass == 2 ? k_index_select<true, 2> :
                      q.pass == 3 ? k_index_select<true, 3> : q.pass == 4 ? k_index_select<true, 4> :
                      q.pass == 5 ? k_index_select<true, 5> : q.pass == 6 ? k_index_select<true, 6> :
                      q.pass == 7 ? k_index_select<true, 7> : q.pass == 8 ? k_index_select<true, 8> :
                      q.pass == 9 ? k_index_select<true, 9> : k_index_select<true, 0>;
        hipError_t e = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
        // the worker modes keep the 16-bit workers of the hot steps behind the bodies
        uint32_t hot = 0;
        const bool worker_pass = q.pass == 4 || q.pass == 5 || q.pass == 8 || q.pass == 9;
        if (worker_pass && ix.hot_worker) hot = ((uint32_t)tv.S * ix.hot_rows * 2u + 15u) & ~15u;
        if (hot + 1024u > lds_bytes - fixed) hot = 0;   // (never with a sensible table; the kernel then must not look for them)
        IndexView ixk = ix;
        if (!hot) ixk.hot_worker = nullptr;
        return launch_kernel(ev, kernel, dim3((unsigned)blocks), dim3((unsigned)kSelThreads), lds_bytes, st, tv, ixk, q,
                             park_mem, lds_bytes - fixed - hot);
    }
    auto kernel = q.pass == 1 ? k_index_select<false, 1> : q.pass == 2 ? k_index_select<false, 2> :
                  q.pass == 3 ? k_index_select<false, 3> : q.pass == 4 ? k_index_select<false, 4> :
                  q.pass == 5 ? k_index_select<false, 5> : q.pass == 6 ? k_index_select<false, 6> :
                  q.pass == 7 ? k_index_select<false, 7> : q.pass == 8 ? k_index_select<false, 8> :
                  q.pass == 9 ? k_index_select<false, 9> : k_index_select<false, 0>;
    return launch_kernel(ev, kernel, dim3((unsigned)blocks), dim3((unsigned)kSelThreads), kLdsCtrlBytes, st, tv, ix, q,
                         park_mem, 0u);
}

}  // namespace infaas
