// Device helpers shared by the lookup kernels: readers of index memory and the search of a body.
#pragma once

#include "internal.h"

namespace infaas {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

#define INFAAS_LDS __attribute__((address_space(3)))

// Workgroup barrier that orders LDS traffic only: what the wavefronts have written to LDS is visible
// to each other behind it, while their requests to global memory stay in flight (__syncthreads also
// waits for those -- for an atomic on a contended word, microseconds).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}


// Readers of index memory by 32-bit byte address: an LDS address, or an offset from a global base.
struct LdsMem {
    __device__ __forceinline__ uint32_t ld32(uint32_t a, uint32_t imm) const { return *(const INFAAS_LDS uint32_t *)(a + imm); }
    __device__ __forceinline__ uint32_t ld16(uint32_t a, uint32_t imm) const { return *(const INFAAS_LDS uint16_t *)(a + imm); }
    __device__ __forceinline__ v2u ld64(uint32_t a) const { return *(const INFAAS_LDS v2u *)a; }
};
struct GlobalMem {
    const uint8_t *p;
    __device__ __forceinline__ uint32_t ld32(uint32_t a, uint32_t imm) const { return *(const uint32_t *)(p + a + imm); }
    __device__ __forceinline__ uint32_t ld16(uint32_t a, uint32_t imm) const { return *(const uint16_t *)(p + a + imm); }
};

// First fitting step of kN bodies (one per query of this lane), as bit sets; the kN searches are
// interleaved so that their dependent reads overlap.  Branch-free apart from the wave-uniform
// probe count.  body[k] / re[k]: address and keys per array (Re) of the body; dd[k]: accuracy
// threshold in key space; lim[k]: latency bound.
template <int kN, class Mem>
__device__ __forceinline__ void search_bodies(const Mem &mem, int nit, const uint32_t (&body)[kN],
                                              const uint32_t (&re)[kN], const uint32_t (&dd)[kN],
                                              const uint32_t (&lim)[kN], uint32_t (&m)[kN])
{
    uint32_t pa[kN], la[kN], pt[kN], lt[kN];
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        pa[k] = body[k];                       // accuracy key j (1-based) at body + 2 + 2j
        la[k] = body[k] + 2u * re[k];          // probes beyond the keys land on the last sentinel
        pt[k] = la[k];                         // latency key j at body + 2 Re + 4j
        lt[k] = pt[k] + 4u * re[k];
    }
#pragma unroll
    for (int it = 4; it >= 0; --it) {
        if (it < nit) {
            uint32_t ca[kN], ct[kN], ka[kN], kt[kN];
#pragma unroll
            for (int k = 0; k < kN; ++k) {   // all reads of a level first, so that they overlap
                ca[k] = pa[k] + (2u << it);
                ct[k] = pt[k] + (4u << it);
                ka[k] = mem.ld16(ca[k] < la[k] ? ca[k] : la[k], 2u);
                kt[k] = mem.ld32(ct[k] < lt[k] ? ct[k] : lt[k], 0u);
            }
#pragma unroll
            for (int k = 0; k < kN; ++k) {
                pa[k] = ka[k] >= dd[k] ? ca[k] : pa[k];
                pt[k] = kt[k] <= lim[k] ? ct[k] : pt[k];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kN; ++k) {
        // A[p] at body + 4 + 6 Re + 4p with pa = body + 2p;  S[ps] at body + 4 + 10 Re + 4 ps with
        // pt = body + 2 Re + 4 ps
        const uint32_t a_at = 2u * pa[k] + (6u * re[k] - body[k]);
        const uint32_t s_at = pt[k] + 8u * re[k];
        m[k] = mem.ld32(a_at, 4u) & mem.ld32(s_at, 4u);
    }
}

// The closest variant of slice (t, b) for a query that nothing satisfies, by the whole wavefront over
// the whole slice in rank order: first by (requirements missed, latency beyond `bound`, accuracy
// below `am`), the earlier rank at a tie.  Entries of a table that serves one state which belong to
// variants of other states (latency key all ones) are passed over.  Returns the caller's row, the
// same in every lane, or -1 when the slice has no entry to offer; *how gets its distance.
struct HowFar {
    int32_t missed;          // of the two requirements
    int64_t over, shortf;    // latency beyond the bound, accuracy below the bound (0 when met)
};
// (requirements missed, latency beyond the bound, accuracy below the bound): the smaller, the closer
__device__ __forceinline__ bool closer_or_equal(const HowFar &a, const HowFar &b)
{
    return a.missed < b.missed || (a.missed == b.missed && (a.over < b.over || (a.over == b.over && a.shortf <= b.shortf)));
}
__device__ __forceinline__ int32_t closest_by_scan(const TableView &tv, int32_t t, int32_t b, int64_t am, int64_t bound, int lane,
                                                   HowFar *how = nullptr)
{
    const int32_t seg = tv.seg_off[t], L = tv.seg_len[t];
    const int64_t col = (int64_t)b * tv.Vp + seg;
    // per lane the best of its entries, earlier rank first
    int32_t b_missed = 3, b_pos = 0x7FFFFFFF;
    int64_t b_over = 0, b_short = 0;
    for (int32_t pos = lane; pos < L; pos += 64) {
        const int64_t tt = (int64_t)tv.tot_r[col + pos], a = (int64_t)tv.acc_r[col + pos];
        const int64_t over = tt > bound ? tt - bound : 0, shortf = a < am ? am - a : 0;
        const int32_t missed = (over > 0) + (shortf > 0);
        const bool masked = tv.state != nullptr && tt == 0xFFFFFFFFll;   // a variant of another state
        const bool better = !masked && (missed < b_missed || (missed == b_missed && (over < b_over ||
                            (over == b_over && shortf < b_short))));
        if (better) { b_missed = missed; b_over = over; b_short = shortf; b_pos = pos; }
    }
    for (int off = 32; off; off >>= 1) {   // then the best of the wavefront
        const int32_t o_missed = __shfl_xor(b_missed, off), o_pos = __shfl_xor(b_pos, off);
        const int64_t o_over = __shfl_xor(b_over, off), o_short = __shfl_xor(b_short, off);
        const bool better = o_missed < b_missed || (o_missed == b_missed && (o_over < b_over ||
                            (o_over == b_over && (o_short < b_short || (o_short == b_short && o_pos < b_pos)))));
        if (better) { b_missed = o_missed; b_over = o_over; b_short = o_short; b_pos = o_pos; }
    }
    if (how) { how->missed = b_missed; how->over = b_over; how->shortf = b_short; }
    return b_missed < 3 ? tv.orig_r[col + b_pos] : -1;
}

// Accuracy bound in key space: keys are acc - acc_base + 1 >= 1, so the bound is
// min_acc - acc_base + 1 limited to [1, 65536] (65536 is above every key).
__device__ __forceinline__ uint32_t acc_threshold(int32_t min_acc, int32_t acc_base_m1)
{
    const int32_t d = __builtin_elementwise_sub_sat(min_acc, acc_base_m1);   // acc_base_m1 = acc_base - 1
    return (uint32_t)(d < 1 ? 1 : (d > 65536 ? 65536 : d));
}

}  // namespace
}  // namespace infaas
