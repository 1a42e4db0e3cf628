// Scaling decision on a change in query load (Section 4.2.2, scaling up): for a running variant,
// its instance count and the incoming load, either nothing, or replicate the variant, or upgrade
// to a variant of the same model architecture with a higher saturation throughput that meets the
// latency objective -- whichever is cheaper by the cost function of the integer program of
// Section 4.2.1, C * (delta + lambda * T_load * max(delta, 0)) summed over the touched variants.
//
// One lane per request.  Per batch size and architecture the library keeps the candidates for an
// upgrade as 16-byte records {throughput, latency, cost of one loaded instance}, sorted by descending
// throughput and without the variants that can never win: v loses to w for every request when w has
// at least v's throughput, at most v's latency and a lower cost per instance (or the same and a lower
// row), because w then passes every test v passes and needs no more instances.  A lane walks its run
// until the throughput drops to the running variant's and keeps the cheapest.  All costs are exact
// integers (times 1,000,000, because lambda is per second and the loading latency in
// microseconds), compared in 128 bits.
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
        const uint32_t *mine = sv.rows + (int64_t)(valid ? cur : 0) * sv.row_words;
        const uint4 head = *(const uint4 *)mine;                        // {throughput, hardware cost, cost of one instance}
        const uint64_t own_unit = ((uint64_t)head.w << 32) | head.z;
        const double own_inv = *(const double *)(mine + 4);
        const int32_t own_lat = (int32_t)mine[kScaleRowLat + (valid ? b : 0)];
        const uint32_t own_qps = head.x;
        const int2 run = *(const int2 *)(mine + sv.pairs_at + 2 * (valid ? b : 0));   // its architecture's list at b
        const uint64_t need = (uint64_t)(uint32_t)load * (uint32_t)sv.slack_pct;   // hundredths of a query per second
        const bool scaling = valid && (uint64_t)own_qps * (uint32_t)n_cur * 100u < need;
        int32_t action = 0, variant = -1, instances = 0;
        if (scaling) {
            // everything is compared with the credit for unloading the running instances added, so
            // that no difference can become negative
            const uint64_t saved = (uint64_t)head.y * (uint32_t)n_cur * 1000000u;   // < 2^61
            bool have = false;
            u128 best = 0;
            int32_t best_at = -1;     // place of the best upgrade in the list, -1: replication is best
            uint32_t best_n = 0;
            if (own_lat <= slo) {   // replicate
                best_n = ceil_div(need, 100u * (uint64_t)own_qps, own_inv) - (uint32_t)n_cur;
                best = (u128)own_unit * best_n + saved;
                have = true;
            }
            // upgrade: the list is read four candidates at a time, so that their loads overlap
            // instead of each waiting for the decision on the one before
            const ScaleCand *list = sv.cand + run.x;                       // run = {first, count}
            const int32_t *list_row = (const int32_t *)(list + run.y);    // the rows sit behind the candidates
            for (int32_t i0 = 0; i0 < run.y; i0 += kChunk) {
                ScaleCand c[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) c[j] = list[i0 + j < run.y ? i0 + j : run.y - 1];
                bool more = true;
#pragma unroll
                for (int j = 0; j < kChunk; ++j) {
                    // descending throughput: nothing from here on supports more than cur
                    more = more && i0 + j < run.y && c[j].qps > own_qps;
                    if (more && c[j].lat <= slo) {
                        const uint64_t per = 100u * (uint64_t)c[j].qps;
                        const uint32_t inst = ceil_div(need, per, 1.0 / (double)per);
                        const u128 cost = (u128)c[j].unit * inst;
                        // replication keeps a tie; among upgrades of equal cost the lower row wins
                        bool better = !have || cost < best;
                        if (cost == best && best_at >= 0) better = list_row[i0 + j] < list_row[best_at];
                        if (better) { best = cost; best_at = i0 + j; best_n = inst; have = true; }
                    }
                }
                if (!more) break;
            }
            action = !have ? 3 : (best_at < 0 ? 1 : 2);
            if (have) {
                variant = best_at < 0 ? cur : list_row[best_at];
                instances = (int32_t)best_n;
            }
        }
        if (in) {
            __builtin_nontemporal_store(action, out_action + r);
            __builtin_nontemporal_store(variant, out_variant + r);
            __builtin_nontemporal_store(instances, out_instances + r);
        }
    }
}

}  // namespace

hipError_t launch_scale(const ScaleView &sv, int64_t R, const int32_t *r_variant, const int32_t *r_instances,
                        const int32_t *r_load_qps, const int32_t *r_slo_us, const int32_t *r_batch_idx,
                        int32_t *out_action, int32_t *out_variant, int32_t *out_instances, int num_cus,
                        hipStream_t st, const LaunchEvents *ev)
{
    if (R <= 0) return hipSuccess;
    const int64_t want = (R + kThreads - 1) / kThreads;
    const int64_t blocks = want < (int64_t)num_cus * 32 ? want : (int64_t)num_cus * 32;
    return launch_kernel(ev, k_scale, dim3((unsigned)blocks), dim3(kThreads), 0, st, sv, R, r_variant, r_instances,
                         r_load_qps, r_slo_us, r_batch_idx, out_action, out_variant, out_instances);
}

}  // namespace infaas
