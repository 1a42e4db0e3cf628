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

// Accuracy bound in key space: keys are acc - acc_base + 1 >= 1, so the bound is
// min_acc - acc_base + 1 limited to [1, 65536] (65536 is above every key).
__device__ __forceinline__ uint32_t acc_threshold(int32_t min_acc, int32_t acc_base_m1)
{
    const int32_t d = __builtin_elementwise_sub_sat(min_acc, acc_base_m1);   // acc_base_m1 = acc_base - 1
    return (uint32_t)(d < 1 ? 1 : (d > 65536 ? 65536 : d));
}

}  // namespace
}  // namespace infaas
