// Scaling decision on a change in query load (Section 4.2.2, scaling up): for a running variant,
// its instance count and the incoming load, either nothing, or replicate the variant, or upgrade
// to a variant of the same model architecture with a higher saturation throughput that meets the
// latency objective -- whichever is cheaper by the cost function of the integer program of
// Section 4.2.1, C * (delta + lambda * T_load * max(delta, 0)) summed over the touched variants.
//
// One lane per request, one cache line per request.  Per batch size and architecture the host keeps
// the candidates for an upgrade sorted by descending throughput and without the variants that can
// never win: v loses to w for every request when w has at least v's throughput, at most v's latency
// and a lower cost per instance (or the same and a lower row), because w then passes every test v
// passes and needs no more instances.  The candidates of a running variant are the prefix of that
// list with a higher throughput than its own; the first five of them are copied, with everything
// else the decision reads about the variant, into a 128-byte block per (batch size, variant), so a
// request costs one uncoalesced line (longer prefixes continue in the shared list).  All costs are
// exact integers (times 1,000,000, because lambda is per second and the loading latency in
// microseconds), compared in 128 bits.
//
// Scaling down (Section 4.2.2, second algorithm) is the same kernel on a second set of blocks: keep,
// or remove one instance when the others still carry the load, or downgrade to a variant of the same
// architecture with a lower hardware cost that meets the latency objective -- whichever lowers the
// same objective most.  There the lists are sorted by ascending hardware cost, the candidates of a
// running variant are the prefix with a lower one, and v loses to w for every request when w
// besides has at most v's hardware cost.
#include "internal.h"

namespace infaas {

namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 4;   // candidates of a list read together
typedef unsigned __int128 u128;

// ceil(need / per) for need < 2^38 and 1 <= per < 2^38 with a quotient below 2^32, given
// per_inv = 1 / per rounded to nearest: need * per_inv is within 2^-51 of the quotient relative to it,
// far less than one unit, so its integer part is the exact floor or one beside it; exact integer
// tests settle which.
__device__ __forceinline__ uint32_t ceil_div(uint64_t need, uint64_t per, double per_inv)
{
    uint32_t q = (uint32_t)((double)need * per_inv);
    uint64_t p = (uint64_t)q * per;
    if (p > need) { q -= 1u; p -= per; }
    else if (p + per <= need) { q += 1u; p += per; }
    return q + (p < need ? 1u : 0u);
}

template <bool kDown>
__global__ __launch_bounds__(kThreads) void k_scale(ScaleView sv, int64_t R, const int32_t *__restrict__ r_variant,
                                                    const int32_t *__restrict__ r_instances,
                                                    const int32_t *__restrict__ r_load_qps,
                                                    const int32_t *__restrict__ r_slo_us,
                                                    const int32_t *__restrict__ r_batch_idx,
                                                    int32_t *__restrict__ out_action, int32_t *__restrict__ out_variant,
                                                    int32_t *__restrict__ out_instances)
{
    for (int64_t r0 = (int64_t)blockIdx.x * kThreads; r0 < R; r0 += (int64_t)gridDim.x * kThreads) {
        const int64_t r = r0 + threadIdx.x;
        const bool in = r < R;
        const int32_t cur = in ? __builtin_nontemporal_load(r_variant + r) : -1;
        const int32_t n_cur = in ? __builtin_nontemporal_load(r_instances + r) : 0;
        const int32_t load = in ? __builtin_nontemporal_load(r_load_qps + r) : 0;
        const int32_t slo = in ? __builtin_nontemporal_load(r_slo_us + r) : 0;
        const int32_t b = in ? __builtin_nontemporal_load(r_batch_idx + r) : 0;
        const bool valid = (uint32_t)cur < (uint32_t)sv.V && (uint32_t)b < (uint32_t)sv.B &&
                           (uint32_t)n_cur <= 1000000u && (uint32_t)load <= 1000000000u;
        // the request's block: one cache line, all of it requested at once
        const uint4 *blk = (const uint4 *)((kDown ? sv.blocks_down : sv.blocks) + ((int64_t)(valid ? b : 0) * sv.V + (valid ? cur : 0)) * kScaleBlockWords);
        const uint4 head = blk[0];      // {throughput, hardware cost, cost of one instance}
        const uint4 more = blk[1];      // {latency, candidates, their list, row of the fifth}
        uint4 slot[kScaleInBlock];
#pragma unroll
        for (int j = 0; j < kScaleInBlock; ++j) slot[j] = blk[2 + j];   // {throughput, latency, cost of one instance}
        const uint4 rows4 = blk[7];
        const int32_t slot_row[kScaleInBlock] = {(int32_t)rows4.x, (int32_t)rows4.y, (int32_t)rows4.z, (int32_t)rows4.w,
                                                 (int32_t)more.w};
        const uint32_t own_qps = head.x;
        const uint64_t own_unit = ((uint64_t)head.w << 32) | head.z;
        const int32_t own_lat = (int32_t)more.x;
        const int32_t m = (int32_t)more.y;
        const uint64_t need = (uint64_t)(uint32_t)load * (uint32_t)sv.slack_pct;   // hundredths of a query per second
        int32_t action = 0, variant = -1, instances = 0;
        // everything is compared with the credit for unloading the running instances added, so
        // that no difference can become negative
        const uint64_t saved = (uint64_t)head.y * (uint32_t)n_cur * 1000000u;   // < 2^61
        bool have = false;
        u128 best = 0;
        int32_t best_row = -1;    // row of the best switch, -1: the running variant is best
        uint32_t best_n = 0;
        // a switch to a candidate (which has a higher throughput, resp. a lower hardware cost, than cur
        // by construction); `floor_n`: the fewest instances a switch loads
        auto offer = [&](uint32_t qps, int32_t lat, uint64_t unit, int32_t row, uint32_t floor_n) {
            if (lat > slo) return;
            const uint64_t per = 100u * (uint64_t)qps;
            uint32_t inst = ceil_div(need, per, 1.0 / (double)per);
            inst = inst < floor_n ? floor_n : inst;
            const u128 cost = (u128)unit * inst;
            // the running variant keeps a tie; among switches of equal cost the lower row wins
            const bool better = !have || cost < best || (cost == best && best_row >= 0 && row < best_row);
            if (better) { best = cost; best_row = row; best_n = inst; have = true; }
        };
        auto offer_all = [&](uint32_t floor_n) {
#pragma unroll
            for (int j = 0; j < kScaleInBlock; ++j)
                if (j < m) offer(slot[j].x, (int32_t)slot[j].y, ((uint64_t)slot[j].w << 32) | slot[j].z, slot_row[j], floor_n);
            if (m > kScaleInBlock) {   // the rest of the prefix from the shared list, four at a time
                const ScaleCand *list = (kDown ? sv.cand_down : sv.cand) + more.z;
                for (int32_t i0 = kScaleInBlock; i0 < m; i0 += kChunk) {
                    ScaleCand c[kChunk];
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) c[j] = list[i0 + j < m ? i0 + j : m - 1];
#pragma unroll
                    for (int j = 0; j < kChunk; ++j)
                        if (i0 + j < m) offer(c[j].qps, c[j].lat, c[j].unit, c[j].row, floor_n);
                }
            }
        };
        if constexpr (!kDown) {
            const bool scaling = valid && (uint64_t)own_qps * (uint32_t)n_cur * 100u < need;
            if (scaling) {
                if (own_lat <= slo) {   // replicate
                    const uint64_t per = 100u * (uint64_t)own_qps;
                    best_n = ceil_div(need, per, 1.0 / (double)per) - (uint32_t)n_cur;
                    best = (u128)own_unit * best_n + saved;
                    have = true;
                }
                offer_all(0u);          // upgrade
                action = !have ? 3 : (best_row < 0 ? 1 : 2);
                if (have) {
                    variant = best_row < 0 ? cur : best_row;
                    instances = (int32_t)best_n;
                }
            }
        } else if (valid) {
            // keeping everything costs `saved` on this scale; removing one instance one hardware cost
            // less, allowed when at least one instance stays and the rest carries the load
            best = saved;
            have = true;
            const bool removable = n_cur >= 2 && (uint64_t)own_qps * (uint32_t)(n_cur - 1) * 100u >= need;
            const bool remove = removable && head.y > 0u;   // (at no hardware cost there is nothing to gain)
            if (remove) best = saved - (uint64_t)head.y * 1000000u;
            offer_all(1u);              // downgrade: at least one instance serves
            if (best_row >= 0) { action = 2; variant = best_row; instances = (int32_t)best_n; }
            else if (remove) { action = 1; variant = cur; instances = 1; }
        }
        if (in) {
            __builtin_nontemporal_store(action, out_action + r);
            __builtin_nontemporal_store(variant, out_variant + r);
            __builtin_nontemporal_store(instances, out_instances + r);
        }
    }
}

}  // namespace

hipError_t launch_scale(const ScaleView &sv, bool down, int64_t R, const int32_t *r_variant, const int32_t *r_instances,
                        const int32_t *r_load_qps, const int32_t *r_slo_us, const int32_t *r_batch_idx,
                        int32_t *out_action, int32_t *out_variant, int32_t *out_instances, int num_cus,
                        hipStream_t st, const LaunchEvents *ev)
{
    if (R <= 0) return hipSuccess;
    const int64_t want = (R + kThreads - 1) / kThreads;
    const int64_t blocks = want < (int64_t)num_cus * 32 ? want : (int64_t)num_cus * 32;
    if (down)
        return launch_kernel(ev, k_scale<true>, dim3((unsigned)blocks), dim3(kThreads), 0, st, sv, R, r_variant,
                             r_instances, r_load_qps, r_slo_us, r_batch_idx, out_action, out_variant, out_instances);
    return launch_kernel(ev, k_scale<false>, dim3((unsigned)blocks), dim3(kThreads), 0, st, sv, R, r_variant, r_instances,
                         r_load_qps, r_slo_us, r_batch_idx, out_action, out_variant, out_instances);
}

}  // namespace infaas
