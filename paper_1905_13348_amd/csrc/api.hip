// Host runtime of libinfaas_sel: handle, variant-store build, scratch, launch sequencing.
// The operation and its C ABI are specified in include/infaas_sel.h.
#include "infaas_sel.h"
#include "internal.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

using namespace infaas;

namespace {

thread_local char g_last_error[320] = "";

// Records which HIP call failed and why; returns true when the call succeeded.
bool hip_ok(hipError_t e, const char *what)
{
    if (e == hipSuccess) return true;
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
    (void)hipGetLastError();
    return false;
}
#define HIP_OK(call) hip_ok((call), #call)

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (!HIP_OK(hipGetDevice(&prev))) { ok = false; return; }
        if (prev != dev && !HIP_OK(hipSetDevice(dev))) ok = false;
        target = dev;
    }
    ~DeviceGuard()
    {
        if (prev >= 0 && prev != target) (void)hipSetDevice(prev);
    }
    int target = -1;
};

struct TimedLaunch {
    int kid;
    hipEvent_t a, b;
};

// ---- scratch memory for infaas_sel_select_noalloc
// The lookup kernel keeps one queue of parked queries per wavefront; every other entry point takes
// them from a hipMalloc'ed block of the handle.  For callers that may not allocate, the same queues
// live in this array, which the code object brings with it: 256 workgroups x 16 wavefronts x 320
// records x 16 bytes.  Every device the library runs on holds its own copy until the process ends.
// Host code never passes the array's name to a kernel (on the host the name is only a stand-in for
// the symbol): static_scratch() looks the device address up once per device and hands that out.
constexpr int kStaticMaxCus = 256;
constexpr size_t kStaticScratchBytes = (size_t)kStaticMaxCus * 16 * 320 * 16;   // 20 MiB
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on device `dev`, which must be the current device.  Null on failure
// (the reason is then in infaas_sel_last_error()).
void *static_scratch(int dev)
{
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

template <typename T>
hipError_t dev_alloc(T **p, size_t count)
{
    *p = nullptr;
    return hipMalloc((void **)p, std::max<size_t>(count, 1) * sizeof(T));
}

}  // namespace

struct infaas_sel {
    int32_t T = 0, B = 0, device = 0;
    uint32_t flags = 0;
    int32_t lds_limit = 4096;
    int num_cus = 256;
    std::vector<int32_t> batch_sizes;

    bool loaded = false;
    // variant store (device)
    int32_t V = 0, Vp = 0;
    int32_t *d_acc = nullptr, *d_queue = nullptr, *d_orig = nullptr, *d_lat = nullptr;
    uint32_t *d_rank = nullptr, *d_perm = nullptr;
    int32_t *d_seg_off = nullptr, *d_seg_len = nullptr, *d_slot_of = nullptr;
    int32_t *d_acc_r = nullptr, *d_lat_r = nullptr, *d_orig_r = nullptr, *d_gpos = nullptr;
    uint32_t *d_tot_r = nullptr;
    int64_t table_bytes = 0;
    int32_t max_segment = 0, max_lds_segment = 0, wide_segments = 0;
    TableView tv{};
    // state-aware selection: this table then serves the Active variants, `inactive` (a handle of
    // its own, built from the same rows) the Inactive ones
    std::vector<int32_t> h_task, h_acc, h_lat;   // host copies of the static columns, for building `inactive`
    int32_t *d_state = nullptr;                  // [Vp] state per slot (see TableView::state)
    infaas_sel *inactive = nullptr;
    int32_t *d_open = nullptr;                   // lists of the queries the Active tier leaves open (grows)
    int32_t *d_open_count = nullptr;             // [workgroups of the lookup kernel]
    int64_t open_queries = 0, open_bytes = 0;    // pass size d_open is good for; its size
    int64_t open_words = 0;                      // 32-bit words of the lists proper; the side lists, if any, follow them
    bool open_side = false;
    // scaling decisions
    ScaleView sv{};
    std::vector<void *> scale_mem;               // the device arrays sv points into
    bool scaling_loaded = false;
    // worker selection (on the handle the caller holds; the step_worker arrays hang off both indexes)
    WorkerView wv{};
    std::vector<void *> worker_mem;              // the device arrays wv points into
    bool workers_loaded = false, workers_dirty = false;
    bool instance_states = false;                // the variants' states follow from their instances' (wv.inst_state)
    bool steps_stale = false;                    // this table's ix.step_worker is older than its index or the workers

    // staircase index
    IndexView ix{};
    bool have_index = false;
    uint32_t index_lds_bytes = 0;     // dynamic LDS of the lookup kernel; 0 = read the index from global memory
    uint32_t ix_stats[kCtlWords] = {0};      // copy of ix.ctrl taken after the build at load time
    std::vector<int32_t> group_task0;        // host copy of ix.group_task0 (empty: one group)
    int64_t ix_bytes = 0, ix_steps = 0;      // pool bytes and steps of the index when it was loaded
    GroupScratch gs{};                       // scratch of the group-by-group selection (grows with the batch)
    int64_t gs_queries = 0, gs_bytes = 0;    // batch size it is good for; its size
    int32_t *d_park = nullptr;        // queues of parked queries of the lookup kernel (fixed size)
    int64_t park_bytes = 0;
    uint32_t *host_stats = nullptr;   // pinned, device-visible: six counters of the latest index build (kCtlMaxK0 .., pool, steps)
    int32_t *static_park = nullptr;   // the same queues inside the library's static device array (may be null)
    const uint32_t *last_stats = nullptr;   // statistics of the most recent lookup launch (this table's or the Inactive tier's)

    // scan scratch
    ScanScratch sc{};
    int64_t sc_capacity = 0;
    int32_t sc_slices = 0;
    int64_t scratch_bytes = 0;
    bool cnt_dirty = false;

    // timing
    bool timing = false;
    std::vector<TimedLaunch> pending;
    std::vector<hipEvent_t> free_events;
    infaas_sel_timings acc{};

    void free_table()
    {
        (void)hipFree(d_acc); (void)hipFree(d_queue); (void)hipFree(d_orig); (void)hipFree(d_lat);
        (void)hipFree(d_rank); (void)hipFree(d_perm); (void)hipFree(d_seg_off);
        (void)hipFree(d_seg_len); (void)hipFree(d_slot_of);
        (void)hipFree(d_acc_r); (void)hipFree(d_lat_r); (void)hipFree(d_orig_r); (void)hipFree(d_gpos);
        (void)hipFree(d_tot_r);
        d_acc = d_queue = d_orig = d_lat = d_seg_off = d_seg_len = d_slot_of = nullptr;
        d_acc_r = d_lat_r = d_orig_r = d_gpos = nullptr;
        d_tot_r = nullptr;
        d_rank = d_perm = nullptr;
        (void)hipFree(d_state);
        d_state = nullptr;
        loaded = false;
        table_bytes = 0;
        for (void *p : scale_mem) (void)hipFree(p);
        scale_mem.clear();
        sv = ScaleView{};
        scaling_loaded = false;
        free_index();
        drop_inactive();
    }
    void drop_inactive();
    void free_index()
    {
        (void)hipFree(ix.pool); (void)hipFree(ix.step_row); (void)hipFree(ix.ctrl);  // hdr lives in pool's allocation
        (void)hipFree(ix.stats); (void)hipFree(ix.slice_room);
        (void)hipFree((void *)ix.task_group); (void)hipFree((void *)ix.group_task0); (void)hipFree(ix.gctrl);
        (void)hipFree(ix.step_worker); (void)hipFree(ix.hot_worker);
        (void)hipFree(d_park);
        d_park = nullptr;
        park_bytes = 0;
        ix = IndexView{};
        group_task0.clear();
        free_group_scratch();
        last_stats = nullptr;
        have_index = false;
        index_lds_bytes = 0;
    }
    void free_group_scratch()
    {
        (void)hipFree(gs.rec); (void)hipFree(gs.perm); (void)hipFree(gs.res); (void)hipFree(gs.desc);
        (void)hipFree(gs.gcount);
        gs = GroupScratch{};
        gs_queries = gs_bytes = 0;
    }
    void free_scratch()
    {
        (void)hipFree(sc.cnt); (void)hipFree(sc.bucket_off); (void)hipFree(sc.cursor);
        (void)hipFree(sc.tile_off); (void)hipFree(sc.wide_off); (void)hipFree(sc.counters);
        (void)hipFree(sc.recs); (void)hipFree(sc.best);
        sc = ScanScratch{};
        sc_capacity = 0;
        sc_slices = 0;
        scratch_bytes = 0;
    }
};

void infaas_sel::drop_inactive()
{
    for (void *p : worker_mem) (void)hipFree(p);
    worker_mem.clear();
    wv = WorkerView{};
    workers_loaded = workers_dirty = instance_states = false;
    (void)hipFree(ix.step_worker); (void)hipFree(ix.hot_worker);
    ix.step_worker = nullptr;
    ix.hot_worker = nullptr;
    (void)hipFree(d_open); (void)hipFree(d_open_count);
    d_open = d_open_count = nullptr;
    open_queries = open_bytes = open_words = 0;
    open_side = false;
    if (inactive) infaas_sel_destroy(inactive);
    inactive = nullptr;
    last_stats = nullptr;
}

namespace {

bool get_event(infaas_sel *h, hipEvent_t *e)
{
    if (!h->free_events.empty()) {
        *e = h->free_events.back();
        h->free_events.pop_back();
        return true;
    }
    return hipEventCreate(e) == hipSuccess;
}

// Hands a launcher the pair of events to attach to its kernel when timing is on.
struct LaunchTimer {
    infaas_sel *h;
    TimedLaunch tl{};
    LaunchEvents pair{};
    bool active = false;
    LaunchTimer(infaas_sel *h_, int kid, hipStream_t) : h(h_)
    {
        if (!h->timing) return;
        tl.kid = kid;
        if (!get_event(h, &tl.a)) return;
        if (!get_event(h, &tl.b)) { h->free_events.push_back(tl.a); return; }
        pair = LaunchEvents{tl.a, tl.b};
        active = true;
    }
    const LaunchEvents *ev() const { return active ? &pair : nullptr; }
    void failed()   // the launch did not happen: the events were never recorded
    {
        if (active) { h->free_events.push_back(tl.a); h->free_events.push_back(tl.b); }
        active = false;
    }
    ~LaunchTimer()
    {
        if (active) h->pending.push_back(tl);
    }
};

int ensure_scratch(infaas_sel *h, int64_t capacity)
{
    const int32_t S = h->T * h->B;
    if (h->sc.recs && h->sc_capacity >= capacity && h->sc_slices == S) return INFAAS_SEL_OK;
    // growing: nothing enqueued earlier may still use the old buffers
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    int64_t cap = std::max<int64_t>(capacity, h->sc_capacity);
    h->free_scratch();
    ScanScratch sc{};
    bool ok = dev_alloc(&sc.cnt, S) == hipSuccess && dev_alloc(&sc.bucket_off, S + 1) == hipSuccess &&
              dev_alloc(&sc.cursor, S) == hipSuccess && dev_alloc(&sc.tile_off, S + 1) == hipSuccess &&
              dev_alloc(&sc.wide_off, S + 1) == hipSuccess && dev_alloc(&sc.counters, 4) == hipSuccess &&
              dev_alloc(&sc.recs, (size_t)cap) == hipSuccess && dev_alloc(&sc.best, (size_t)cap) == hipSuccess;
    h->sc = sc;
    if (!ok) {
        h->free_scratch();
        (void)hipGetLastError();
        return INFAAS_SEL_ERR_OOM;
    }
    if (!HIP_OK(hipMemset(sc.cnt, 0, std::max<size_t>(S, 1) * 4)) ||
        !HIP_OK(hipMemset(sc.counters, 0, 16))) {
        h->free_scratch();
        return INFAAS_SEL_ERR_HIP;
    }
    h->cnt_dirty = false;
    h->sc_capacity = cap;
    h->sc_slices = S;
    h->scratch_bytes = (int64_t)S * 4 * 5 + 8 + 16 + cap * (16 + 4);
    return INFAAS_SEL_OK;
}

constexpr uint32_t kLdsMax = 160 * 1024;  // dynamic LDS the lookup kernel may ask for

constexpr uint32_t kGroupRegionBytes = 144 * 1024;   // a group's bodies: what one LDS holds next to its slices' headers
constexpr uint32_t kGroupMaxSlices = 1900;           // ... 8 bytes of header each
constexpr uint32_t kGroupStepCap = 16384;            // entries of step_row per group (a region holds at most 10,532 steps)
constexpr int32_t kGroupMaxGroups = 120;
constexpr int32_t kGroupMaxTasks = 16384;            // the binning kernel keeps the group of every task in LDS
constexpr uint32_t kGroupHotRows = 8;

// Starting values of the allocator counters and the statistics, then one build, then the counters back.
int build_index_now(infaas_sel *h)
{
    IndexView &ix = h->ix;
    const bool grouped = ix.num_groups > 1;
    uint32_t ctrl0[kCtlWords] = {0};
    ctrl0[kCtlPool] = ctrl0[kCtlPool0] = grouped ? ix.num_groups * ix.region_bytes : kDummyBodyBytes;
    ctrl0[kCtlSteps] = ctrl0[kCtlSteps0] = grouped ? ix.num_groups * ix.group_step_cap : 1u;
    ctrl0[kCtlMaxK0] = 1u;
    ctrl0[kCtlEpoch] = 1u;   // (slice_room is cleared below: build number 0)
    std::vector<uint32_t> g0;
    for (uint32_t g = 0; grouped && g < ix.num_groups; ++g) { g0.push_back(kDummyBodyBytes); g0.push_back(g == 0 ? 1u : 0u); }
    if (!HIP_OK(hipMemcpy(ix.ctrl, ctrl0, sizeof(ctrl0), hipMemcpyHostToDevice)) ||
        !HIP_OK(hipMemset(ix.slice_room, 0, (size_t)h->T * h->B * sizeof(unsigned long long))) ||
        (grouped && !HIP_OK(hipMemcpy(ix.gctrl, g0.data(), g0.size() * 4, hipMemcpyHostToDevice))) ||
        !HIP_OK(launch_index_build(h->tv, ix, nullptr)) || !HIP_OK(hipDeviceSynchronize()) ||
        !HIP_OK(hipMemcpy(h->ix_stats, ix.ctrl, sizeof(ctrl0), hipMemcpyDeviceToHost)))
        return INFAAS_SEL_ERR_HIP;
    // what the selections' first kernels keep up to date from now on
    if (h->host_stats) {
        void *dev = nullptr;
        for (int i = 0; i < 4; ++i) h->host_stats[i] = h->ix_stats[kCtlMaxK0 + i];
        h->host_stats[4] = h->ix_stats[kCtlPool];
        h->host_stats[5] = h->ix_stats[kCtlSteps];
        if (hipHostGetDevicePointer(&dev, h->host_stats, 0) == hipSuccess) {
            h->tv.stat_src = ix.ctrl;
            h->tv.stat_dst = (uint32_t *)dev;
        } else {
            (void)hipGetLastError();
        }
    }
    // bytes and steps of the index as a whole (info only)
    h->ix_bytes = h->ix_stats[kCtlPool];
    h->ix_steps = (int64_t)h->ix_stats[kCtlSteps] - 1;   // (entry 0 of step_row is unused)
    if (grouped) {
        if (!HIP_OK(hipMemcpy(g0.data(), ix.gctrl, g0.size() * 4, hipMemcpyDeviceToHost))) return INFAAS_SEL_ERR_HIP;
        h->ix_bytes -= (int64_t)ix.num_groups * ix.region_bytes;
        h->ix_steps -= (int64_t)ix.num_groups * ix.group_step_cap;
        for (uint32_t g = 0; g < ix.num_groups; ++g) { h->ix_bytes += g0[2 * g]; h->ix_steps += g0[2 * g + 1]; }
    }
    return INFAAS_SEL_OK;
}

// Allocate the staircase index for the loaded table, build it and read its sizes back.
int create_index(infaas_sel *h)
{
    const int64_t S = (int64_t)h->T * h->B;
    const uint32_t worst = 2 * body_bytes(body_re(kBodySteps)) + 2 * (kBodySteps + 1);
    // The build takes room with one add on a pair of 32-bit counters; their sums must not carry.
    // A table with that many slices (millions) gets no index and is answered by the scan engine.
    const int64_t regions = (int64_t)kGroupMaxGroups * kGroupRegionBytes, region_steps = (int64_t)kGroupMaxGroups * kGroupStepCap;
    if (regions + kDummyBodyBytes + S * worst > 0xFFFF0000ll || region_steps + 1 + S * kIndexCap > 0xFFFF0000ll) return INFAAS_SEL_OK;
    IndexView ix{};
    ix.num_groups = 1;
    // room for the regions of a grouped layout in front of what an ungrouped one needs
    ix.pool_bytes = (uint32_t)std::min<int64_t>(regions + kDummyBodyBytes + S * worst + 64, (int64_t)3 << 30);
    ix.step_cap = (uint32_t)std::min<int64_t>(region_steps + 1 + S * kIndexCap, (int64_t)1 << 29);
    // one allocation: the pool, then the headers, so that one 32-bit offset reaches both
    ix.pool_bytes &= ~15u;
    const size_t nstats = (size_t)index_select_blocks(h->num_cus) * kLookupStats;
    bool ok = dev_alloc(&ix.pool, (size_t)ix.pool_bytes + (size_t)(S + 1) * 16) == hipSuccess &&
              dev_alloc(&ix.step_row, ix.step_cap) == hipSuccess && dev_alloc(&ix.ctrl, kCtlWords) == hipSuccess &&
              dev_alloc(&ix.stats, nstats) == hipSuccess && dev_alloc(&ix.gctrl, 2 * (size_t)kGroupMaxGroups) == hipSuccess &&
              dev_alloc(&ix.slice_room, (size_t)S) == hipSuccess;
    ix.hdr = ok ? (uint4 *)(ix.pool + ix.pool_bytes) : nullptr;
    h->ix = ix;
    const size_t park = index_park_bytes(h->num_cus);
    ok = ok && dev_alloc(&h->d_park, park / 4) == hipSuccess;
    h->park_bytes = ok ? (int64_t)park : 0;
    if (!ok) {
        h->free_index();
        (void)hipGetLastError();
        return INFAAS_SEL_ERR_OOM;
    }
    // dummy body of a slice without steps (sentinels only) at offset 0; step_row[0] is never an answer
    uint8_t dummy[kDummyBodyBytes] = {0};
    for (uint32_t i = 8; i < 16; ++i) dummy[i] = 0xFF;  // latency sentinels of the empty body (Re = 2)
    const int32_t none = -1;
    const uint32_t empty_hdr[4] = {0u, kEmptyHdrY, 0u, 4u + body_bytes(2)};
    if (!HIP_OK(hipMemset(ix.stats, 0, nstats * 4)) ||
        !HIP_OK(hipMemcpy(ix.pool, dummy, sizeof(dummy), hipMemcpyHostToDevice)) ||
        !HIP_OK(hipMemcpy(ix.step_row, &none, 4, hipMemcpyHostToDevice)) ||
        !HIP_OK(hipMemcpy(&ix.hdr[S], empty_hdr, sizeof(empty_hdr), hipMemcpyHostToDevice)) ||
        build_index_now(h) != INFAAS_SEL_OK) {
        h->free_index();
        return INFAAS_SEL_ERR_HIP;
    }
    h->have_index = true;
    const int64_t fixed = kLdsCtrlBytes + lds_header_bytes((int32_t)S) + 16;
    const int64_t need = fixed + h->ix_stats[kCtlPool];
    // The lookup kernel mirrors the index in LDS when the slice headers leave at least half of it to
    // the bodies; bodies that do not fit stay in global memory and their queries take the slower
    // path inside the same kernel.  With more headers than that the kernel reads everything from
    // global memory.
    h->index_lds_bytes = fixed <= (int64_t)kLdsMax / 2 ? kLdsMax : 0u;
    // 2 bytes of a step's caller row sit in front of its body, the bits above in a 14-bit header field
    const uint32_t row_bits = h->V > 1 ? 64u - (uint32_t)__builtin_clzll((unsigned long long)(h->V - 1)) : 1u;
    h->ix.row_hi_bits = row_bits > 16 ? row_bits - 16 : 0u;
    const uint32_t hot_max = std::min<uint32_t>(h->ix.row_hi_bits ? kRowHiField / h->ix.row_hi_bits : (uint32_t)kBodySteps, kBodySteps);
    if (need > 2 * (int64_t)kLdsMax && h->T <= kGroupMaxTasks) {
        // Not even half of the bodies fit one LDS: deal the tasks, in order, to groups whose bodies do (with a
        // fifth of the region left free, because staircases grow and shrink with the load), and build
        // again with one region of the pool per group.  Large batches of queries are then binned by
        // group and looked up group by group, every workgroup with its group's bodies in LDS.
        std::vector<uint32_t> hdr((size_t)S * 4);
        if (!HIP_OK(hipMemcpy(hdr.data(), h->ix.hdr, (size_t)S * 16, hipMemcpyDeviceToHost))) { h->free_index(); return INFAAS_SEL_ERR_HIP; }
        const uint32_t hot = std::min(kGroupHotRows, hot_max) & ~1u;
        const uint32_t target = (kGroupRegionBytes - kDummyBodyBytes) / 5 * 4;
        std::vector<uint16_t> task_group((size_t)h->T);
        std::vector<int32_t> task0{0};
        uint32_t bytes = 0, slices = 0;
        for (int32_t t = 0; t < h->T; ++t) {
            uint32_t tb = 0;
            for (int32_t b = 0; b < h->B; ++b) {
                const uint32_t *e = &hdr[((size_t)t * h->B + b) * 4];   // {body address, y, first step, end of bodies}
                if (e[0] != 0u) tb += e[3] - (e[0] + 4u) + 2u * hot + 4u;   // bodies, and room for the first steps' rows
            }
            if (slices > 0 && (bytes + tb > target || slices + (uint32_t)h->B > kGroupMaxSlices)) {
                task0.push_back(t);
                bytes = slices = 0;
            }
            bytes += tb; slices += (uint32_t)h->B;
            task_group[(size_t)t] = (uint16_t)(task0.size() - 1);
        }
        task0.push_back(h->T);
        const int32_t G = (int32_t)task0.size() - 1;
        if (G > 1 && G <= kGroupMaxGroups && (uint32_t)h->B <= kGroupMaxSlices) {
            uint16_t *d_tg = nullptr;
            int32_t *d_t0 = nullptr;
            if (dev_alloc(&d_tg, (size_t)h->T) != hipSuccess || dev_alloc(&d_t0, (size_t)G + 1) != hipSuccess) {
                (void)hipFree(d_tg); (void)hipFree(d_t0); (void)hipGetLastError();
                h->free_index();
                return INFAAS_SEL_ERR_OOM;
            }
            h->ix.task_group = d_tg; h->ix.group_task0 = d_t0;
            h->ix.num_groups = (uint32_t)G; h->ix.region_bytes = kGroupRegionBytes; h->ix.group_step_cap = kGroupStepCap;
            h->ix.hot_rows = hot;
            bool up = HIP_OK(hipMemcpy(d_tg, task_group.data(), (size_t)h->T * 2, hipMemcpyHostToDevice)) &&
                      HIP_OK(hipMemcpy(d_t0, task0.data(), ((size_t)G + 1) * 4, hipMemcpyHostToDevice));
            for (int32_t g = 1; up && g < G; ++g)   // every region begins with the dummy body
                up = HIP_OK(hipMemcpy(h->ix.pool + (size_t)g * kGroupRegionBytes, dummy, sizeof(dummy), hipMemcpyHostToDevice));
            if (!up || build_index_now(h) != INFAAS_SEL_OK) { h->free_index(); return INFAAS_SEL_ERR_HIP; }
            h->group_task0.assign(task0.begin(), task0.end());
            return INFAAS_SEL_OK;
        }
    }
    // LDS left over holds the caller rows of the first steps of every slice (the steps most answers
    // come from), which saves those answers a gather from global memory.  Rebuild with that many.
    const int64_t spare = (int64_t)kLdsMax - need - 1024;   // keep room for staircases that grow with load
    const uint32_t hot = spare > 0 ? (uint32_t)std::min<int64_t>((spare / (4 * S)) * 2, hot_max) : 0u;
    if (h->index_lds_bytes && hot > 0) {
        h->ix.hot_rows = hot;
        if (build_index_now(h) != INFAAS_SEL_OK) {
            h->free_index();
            return INFAAS_SEL_ERR_HIP;
        }
    }
    return INFAAS_SEL_OK;
}

// Lists for the queries that the first tier of a state-aware pass over up to n queries leaves open.
// side: also the lists of the first tier's suggestions beside them (complete Case I), the same size again.
int ensure_open(infaas_sel *h, int64_t n, bool side)
{
    if (h->d_open && h->open_queries >= n && (h->open_side || !side)) return INFAAS_SEL_OK;
    n = std::max(n, h->open_queries);
    side = side || h->open_side;
    // growing: nothing enqueued earlier may still use the old lists
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    (void)hipFree(h->d_open);
    h->d_open = nullptr;
    h->open_queries = h->open_bytes = 0;
    const int blocks = index_select_blocks(h->num_cus);
    h->open_side = false;
    const size_t words = (size_t)blocks * (size_t)index_open_cap((int32_t)n, h->num_cus) * 4;
    if (!h->d_open_count && dev_alloc(&h->d_open_count, (size_t)blocks) != hipSuccess) return INFAAS_SEL_ERR_OOM;
    if (dev_alloc(&h->d_open, words * (side ? 2 : 1)) != hipSuccess) return INFAAS_SEL_ERR_OOM;
    h->open_queries = n;
    h->open_words = (int64_t)words;
    h->open_side = side;
    h->open_bytes = (int64_t)words * 4 * (side ? 2 : 1);
    return INFAAS_SEL_OK;
}

// One pass of the index engine over n <= 2^28 queries.
int index_pass(infaas_sel *h, const QueryView &q, hipStream_t st)
{
    LaunchTimer t(h, INFAAS_SEL_K_INDEX_SELECT, st);
    if (!HIP_OK(launch_index_select(h->tv, h->ix, q, h->d_park, h->index_lds_bytes, h->num_cus, st, t.ev())))
        return INFAAS_SEL_ERR_HIP;
    return INFAAS_SEL_OK;
}

// Below this many queries a call is answered by the one-kernel lookup even when the index is laid
// out in groups: the four launches of the group-by-group path cost more than they save.
constexpr int64_t kGroupMinQueries = (int64_t)1 << 20;

// Scratch of the group-by-group selection for batches of up to n queries.
int ensure_group_scratch(infaas_sel *h, int64_t n)
{
    if (h->gs.rec && h->gs_queries >= n) return INFAAS_SEL_OK;
    // growing: nothing enqueued earlier may still use the old buffers
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    h->free_group_scratch();
    const int64_t tiles = (n + kGroupTile - 1) / kGroupTile, padded = tiles * kGroupTile;
    const size_t G1 = (size_t)h->ix.num_groups + 1;
    GroupScratch gs{};
    bool ok = dev_alloc(&gs.rec, (size_t)padded) == hipSuccess && dev_alloc(&gs.perm, (size_t)padded) == hipSuccess &&
              dev_alloc(&gs.res, (size_t)padded) == hipSuccess && dev_alloc(&gs.desc, (size_t)tiles * G1) == hipSuccess &&
              dev_alloc(&gs.gcount, G1) == hipSuccess;
    h->gs = gs;
    if (!ok) {
        h->free_group_scratch();
        (void)hipGetLastError();
        return INFAAS_SEL_ERR_OOM;
    }
    if (!HIP_OK(hipMemset(gs.gcount, 0, G1 * 4))) { h->free_group_scratch(); return INFAAS_SEL_ERR_HIP; }
    int32_t most = 0;
    for (size_t g = 0; g + 1 < h->group_task0.size(); ++g) most = std::max(most, (h->group_task0[g + 1] - h->group_task0[g]) * h->B);
    h->gs.max_group_slices = most;
    h->gs.stat_blocks = index_select_blocks(h->num_cus);
    h->gs_queries = padded;
    h->gs_bytes = padded * 14 + (int64_t)tiles * (int64_t)G1 * 4;
    return INFAAS_SEL_OK;
}

bool use_groups(const infaas_sel *h, int64_t n)
{
    return h->have_index && h->ix.num_groups > 1 && n >= kGroupMinQueries && (int)h->ix.num_groups <= h->num_cus &&
           group_bin_lds_bytes(h->T, (int32_t)h->ix.num_groups) <= 64 * 1024;
}

// One pass of the group-by-group selection over n <= 2^28 queries (scratch must be there).
int group_pass(infaas_sel *h, const QueryView &q, hipStream_t st)
{
    {
        LaunchTimer t(h, INFAAS_SEL_K_GROUP_BIN, st);
        if (!HIP_OK(launch_group_bin(h->tv, h->ix, q, h->gs, h->num_cus, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    {
        LaunchTimer t(h, INFAAS_SEL_K_GROUP_LOOKUP, st);
        if (!HIP_OK(launch_group_lookup(h->tv, h->ix, q, h->gs, h->num_cus, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    LaunchTimer t(h, INFAAS_SEL_K_GROUP_FINISH, st);
    if (!HIP_OK(launch_group_finish(h->tv, h->ix, q, h->gs, h->num_cus, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    return INFAAS_SEL_OK;
}

bool use_index(infaas_sel *h)
{
    const uint32_t engine = h->flags & INFAAS_SEL_ENGINE_MASK;
    if (!h->have_index || engine == INFAAS_SEL_ENGINE_SCAN) return false;
    if (engine == INFAAS_SEL_ENGINE_INDEX) return true;
    // The first kernel of every selection copies four counters of the latest index build into pinned
    // host memory (TableView::stat_dst), so what is read here is at most one call behind, and no
    // call ever waits for it.
    uint32_t trunc = h->ix_stats[kCtlTrunc], nobody = h->ix_stats[kCtlNoBody];
    if (h->host_stats) {
        trunc = ((volatile uint32_t *)h->host_stats)[kCtlTrunc - kCtlMaxK0];
        nobody = ((volatile uint32_t *)h->host_stats)[kCtlNoBody - kCtlMaxK0];
    }
    // auto: the index (mirrored in LDS when it fits, read from global memory otherwise), unless
    // more than half of the slices could not be indexed completely when the table was loaded or, as
    // far as is known by now, when the index was last rebuilt -- their queries would mostly end in
    // the in-kernel scan, which the bucketed scan engine does faster
    const int64_t S = (int64_t)h->T * h->B;
    return 2 * ((int64_t)trunc + nobody) <= S;
}

// One pass of the scan engine over n <= 2^28 queries.
int scan_pass(infaas_sel *h, const QueryView &q, hipStream_t st)
{
    if (h->cnt_dirty) {  // an earlier call failed between histogram and plan
        if (!HIP_OK(hipStreamSynchronize(st))) return INFAAS_SEL_ERR_HIP;
        if (!HIP_OK(hipMemset(h->sc.cnt, 0, (size_t)h->tv.S * 4))) return INFAAS_SEL_ERR_HIP;
        h->cnt_dirty = false;
    }
    h->cnt_dirty = true;
    {
        LaunchTimer t(h, INFAAS_SEL_K_HISTOGRAM, st);
        if (!HIP_OK(launch_histogram(h->tv, q, h->sc, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    {
        LaunchTimer t(h, INFAAS_SEL_K_PLAN, st);
        if (!HIP_OK(launch_plan(h->tv, h->sc, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    h->cnt_dirty = false;
    const bool wide = h->wide_segments > 0;
    {
        LaunchTimer t(h, INFAAS_SEL_K_SCATTER, st);
        if (!HIP_OK(launch_scatter(h->tv, q, h->sc, wide, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    if (h->max_lds_segment > 0) {
        LaunchTimer t(h, INFAAS_SEL_K_SCAN_LDS, st);
        if (!HIP_OK(launch_scan_lds(h->tv, q, h->sc, h->max_lds_segment, h->num_cus, st, t.ev())))
            return INFAAS_SEL_ERR_HIP;
    }
    if (wide) {
        {
            LaunchTimer t(h, INFAAS_SEL_K_SCAN_WIDE, st);
            if (!HIP_OK(launch_scan_wide(h->tv, q, h->sc, h->num_cus, st, t.ev())))
                return INFAAS_SEL_ERR_HIP;
        }
        LaunchTimer t(h, INFAAS_SEL_K_FINISH_WIDE, st);
        if (!HIP_OK(launch_finish_wide(h->tv, q, h->sc, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    return INFAAS_SEL_OK;
}

constexpr int64_t kMaxPass = (int64_t)1 << 28;
// State-aware selection: 16 bytes of list memory per query of a pass, hence shorter passes.
constexpr int64_t kMaxTierPass = (int64_t)1 << 26;

}  // namespace

extern "C" {

const char *infaas_sel_last_error(void) { return g_last_error; }

const char *infaas_sel_strerror(int status)
{
    switch (status) {
    case INFAAS_SEL_OK: return "ok";
    case INFAAS_SEL_ERR_INVALID_ARG: return "invalid argument";
    case INFAAS_SEL_ERR_NOT_LOADED: return "no variant table loaded";
    case INFAAS_SEL_ERR_OUT_OF_RANGE: return "table value out of range";
    case INFAAS_SEL_ERR_HIP: return "HIP runtime error";
    case INFAAS_SEL_ERR_OOM: return "out of memory";
    default: return "unknown status";
    }
}

int infaas_sel_create(const infaas_sel_config *cfg, infaas_sel_t **out)
{
    if (!cfg || !out) return INFAAS_SEL_ERR_INVALID_ARG;
    if (cfg->num_tasks < 1 || cfg->num_batch_sizes < 1 || cfg->num_batch_sizes > 64)
        return INFAAS_SEL_ERR_INVALID_ARG;
    if ((int64_t)cfg->num_tasks * cfg->num_batch_sizes > ((int64_t)1 << 24))
        return INFAAS_SEL_ERR_INVALID_ARG;
    uint32_t engine = cfg->flags & INFAAS_SEL_ENGINE_MASK;
    if ((cfg->flags & ~INFAAS_SEL_ENGINE_MASK) != 0 || engine > INFAAS_SEL_ENGINE_INDEX)
        return INFAAS_SEL_ERR_INVALID_ARG;
    int32_t lim = cfg->lds_segment_limit == 0 ? 4096 : cfg->lds_segment_limit;
    if (lim < 64 || lim > 8192) return INFAAS_SEL_ERR_INVALID_ARG;
    lim &= ~63;
    int ndev = 0;
    if (!HIP_OK(hipGetDeviceCount(&ndev))) return INFAAS_SEL_ERR_HIP;
    if (cfg->device < 0 || cfg->device >= ndev) return INFAAS_SEL_ERR_INVALID_ARG;

    infaas_sel *h = new (std::nothrow) infaas_sel();
    if (!h) return INFAAS_SEL_ERR_OOM;
    h->T = cfg->num_tasks;
    h->B = cfg->num_batch_sizes;
    h->device = cfg->device;
    h->flags = cfg->flags;
    h->lds_limit = lim;
    if (cfg->batch_sizes) h->batch_sizes.assign(cfg->batch_sizes, cfg->batch_sizes + h->B);
    hipDeviceProp_t prop;
    if (!HIP_OK(hipGetDeviceProperties(&prop, h->device))) {
        delete h;
        return INFAAS_SEL_ERR_HIP;
    }
    h->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    {
        DeviceGuard g(h->device);
        if (g.ok && hipHostMalloc((void **)&h->host_stats, 64, hipHostMallocMapped) != hipSuccess) {
            (void)hipGetLastError();
            h->host_stats = nullptr;
        }
    }
    {
        // address of the static scratch array on this device, for infaas_sel_select_noalloc (a
        // failure here only makes that one call unavailable)
        DeviceGuard g(h->device);
        if (g.ok) h->static_park = (int32_t *)static_scratch(h->device);
    }
    *out = h;
    return INFAAS_SEL_OK;
}

int infaas_sel_load_variants(infaas_sel_t *h, int32_t V, const int32_t *task_id,
                             const int32_t *acc_bp, const int32_t *lat_us, const int32_t *cost,
                             const int32_t *queue_us)
{
    if (!h || V < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (V > 0 && (!task_id || !acc_bp || !lat_us || !cost || !queue_us))
        return INFAAS_SEL_ERR_INVALID_ARG;
    const int32_t T = h->T, B = h->B;

    // ---- validate ranges before touching the old table
    for (int64_t v = 0; v < V; ++v) {
        if (task_id[v] < 0 || task_id[v] >= T || queue_us[v] < 0) return INFAAS_SEL_ERR_OUT_OF_RANGE;
        for (int32_t b = 0; b < B; ++b)
            if (lat_us[v * B + b] < 0 || cost[v * B + b] < 0) return INFAAS_SEL_ERR_OUT_OF_RANGE;
    }

    std::vector<int32_t> keep_task(task_id, task_id + V), keep_acc(acc_bp, acc_bp + V),
        keep_lat(lat_us, lat_us + (size_t)V * B);

    // ---- group rows by task (stable), pad every segment to a multiple of 4 slots
    std::vector<int32_t> seg_len(T, 0), seg_off((size_t)T + 1, 0);
    for (int64_t v = 0; v < V; ++v) seg_len[task_id[v]] += 1;
    int64_t total = 0;
    int32_t max_seg = 0, max_lds_seg = 0, wide = 0;
    for (int32_t t = 0; t < T; ++t) {
        seg_off[t] = (int32_t)total;
        total += (seg_len[t] + 3) & ~3;
        if (total > INT32_MAX - 64) return INFAAS_SEL_ERR_INVALID_ARG;
        max_seg = std::max(max_seg, seg_len[t]);
        if (seg_len[t] > h->lds_limit) wide += 1;
        else max_lds_seg = std::max(max_lds_seg, seg_len[t]);
    }
    seg_off[T] = (int32_t)total;
    const int32_t Vp = (int32_t)((total + 63) & ~(int64_t)63) + 64;

    std::vector<int32_t> acc(Vp, INT32_MIN), queue(Vp, INT32_MAX), orig(Vp, -1), slot_of(std::max(V, 1), 0);
    std::vector<int32_t> lat((size_t)B * Vp, INT32_MAX);
    std::vector<uint32_t> rank((size_t)B * Vp, kNoRank), perm((size_t)B * Vp, 0u);
    std::vector<int32_t> acc_r((size_t)B * Vp, INT32_MIN), lat_r((size_t)B * Vp, 0), orig_r((size_t)B * Vp, -1);
    std::vector<int32_t> gpos((size_t)B * Vp, 0);
    std::vector<uint32_t> tot_r((size_t)B * Vp, 0xFFFFFFFFu);
    {
        std::vector<int32_t> fill(T, 0);
        for (int64_t v = 0; v < V; ++v) {
            int32_t t = task_id[v];
            int32_t slot = seg_off[t] + fill[t]++;
            acc[slot] = acc_bp[v];
            queue[slot] = queue_us[v];
            orig[slot] = (int32_t)v;
            slot_of[v] = slot;
            for (int32_t b = 0; b < B; ++b) lat[(size_t)b * Vp + slot] = lat_us[v * B + b];
        }
    }
    // ---- rank of every row inside its (task, batch) slice under (cost, latency, row)
    {
        std::vector<int32_t> ord;
        for (int32_t t = 0; t < T; ++t) {
            const int32_t L = seg_len[t], seg = seg_off[t];
            if (L == 0) continue;
            ord.resize(L);
            for (int32_t b = 0; b < B; ++b) {
                std::iota(ord.begin(), ord.end(), 0);
                std::sort(ord.begin(), ord.end(), [&](int32_t x, int32_t y) {
                    const int64_t vx = orig[seg + x], vy = orig[seg + y];
                    const int32_t cx = cost[vx * B + b], cy = cost[vy * B + b];
                    if (cx != cy) return cx < cy;
                    const int32_t lx = lat_us[vx * B + b], ly = lat_us[vy * B + b];
                    if (lx != ly) return lx < ly;
                    return vx < vy;
                });
                for (int32_t r = 0; r < L; ++r) {
                    const size_t g = (size_t)b * Vp + seg + r, sl = (size_t)b * Vp + seg + ord[r];
                    perm[g] = (uint32_t)ord[r];
                    rank[sl] = (uint32_t)r;
                    acc_r[g] = acc[seg + ord[r]];
                    lat_r[g] = lat[sl];
                    tot_r[g] = (uint32_t)lat[sl] + (uint32_t)queue[seg + ord[r]];
                    orig_r[g] = orig[seg + ord[r]];
                    gpos[sl] = seg + r;
                }
            }
        }
    }

    // ---- upload
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    h->free_table();
    bool ok = dev_alloc(&h->d_acc, Vp) == hipSuccess && dev_alloc(&h->d_queue, Vp) == hipSuccess &&
              dev_alloc(&h->d_orig, Vp) == hipSuccess && dev_alloc(&h->d_lat, (size_t)B * Vp) == hipSuccess &&
              dev_alloc(&h->d_rank, (size_t)B * Vp) == hipSuccess &&
              dev_alloc(&h->d_perm, (size_t)B * Vp) == hipSuccess &&
              dev_alloc(&h->d_seg_off, (size_t)T + 1) == hipSuccess && dev_alloc(&h->d_seg_len, T) == hipSuccess &&
              dev_alloc(&h->d_slot_of, std::max(V, 1)) == hipSuccess &&
              dev_alloc(&h->d_acc_r, (size_t)B * Vp) == hipSuccess && dev_alloc(&h->d_lat_r, (size_t)B * Vp) == hipSuccess &&
              dev_alloc(&h->d_orig_r, (size_t)B * Vp) == hipSuccess && dev_alloc(&h->d_gpos, (size_t)B * Vp) == hipSuccess &&
              dev_alloc(&h->d_tot_r, (size_t)B * Vp) == hipSuccess;
    if (!ok) {
        h->free_table();
        (void)hipGetLastError();
        return INFAAS_SEL_ERR_OOM;
    }
    auto up = [](void *d, const void *s, size_t bytes) {
        return bytes == 0 || HIP_OK(hipMemcpy(d, s, bytes, hipMemcpyHostToDevice));
    };
    ok = up(h->d_acc, acc.data(), (size_t)Vp * 4) && up(h->d_queue, queue.data(), (size_t)Vp * 4) &&
         up(h->d_orig, orig.data(), (size_t)Vp * 4) && up(h->d_lat, lat.data(), (size_t)B * Vp * 4) &&
         up(h->d_rank, rank.data(), (size_t)B * Vp * 4) && up(h->d_perm, perm.data(), (size_t)B * Vp * 4) &&
         up(h->d_seg_off, seg_off.data(), ((size_t)T + 1) * 4) && up(h->d_seg_len, seg_len.data(), (size_t)T * 4) &&
         up(h->d_slot_of, slot_of.data(), (size_t)std::max(V, 1) * 4) &&
         up(h->d_acc_r, acc_r.data(), (size_t)B * Vp * 4) && up(h->d_lat_r, lat_r.data(), (size_t)B * Vp * 4) &&
         up(h->d_orig_r, orig_r.data(), (size_t)B * Vp * 4) && up(h->d_gpos, gpos.data(), (size_t)B * Vp * 4) &&
         up(h->d_tot_r, tot_r.data(), (size_t)B * Vp * 4);
    if (!ok) {
        h->free_table();
        return INFAAS_SEL_ERR_HIP;
    }
    h->V = V;
    h->Vp = Vp;
    h->max_segment = max_seg;
    h->max_lds_segment = max_lds_seg;
    h->wide_segments = wide;
    h->table_bytes = (int64_t)Vp * 4 * (3 + 8 * (int64_t)B) + ((int64_t)2 * T + 1 + std::max(V, 1)) * 4;
    TableView tv{};
    tv.T = T; tv.B = B; tv.S = T * B; tv.V = V; tv.Vp = Vp; tv.lds_limit = h->lds_limit;
    tv.acc = h->d_acc; tv.queue = h->d_queue; tv.orig = h->d_orig; tv.lat = h->d_lat;
    tv.rank = h->d_rank; tv.perm = h->d_perm; tv.seg_off = h->d_seg_off; tv.seg_len = h->d_seg_len;
    tv.slot_of = h->d_slot_of;
    tv.acc_r = h->d_acc_r; tv.tot_r = h->d_tot_r; tv.lat_r = h->d_lat_r; tv.orig_r = h->d_orig_r;
    tv.gpos = h->d_gpos;
    tv.acc_base = 0;
    for (int64_t v = 0; v < V; ++v) tv.acc_base = (v == 0 || acc_bp[v] < tv.acc_base) ? acc_bp[v] : tv.acc_base;
    // the lookup forms acc_base - 1; a slice that holds the one accuracy below this base is not indexed
    if (tv.acc_base == INT32_MIN) tv.acc_base = INT32_MIN + 1;
    tv.state = nullptr;
    tv.want_state = 1;
    h->tv = tv;
    h->h_task.swap(keep_task); h->h_acc.swap(keep_acc); h->h_lat.swap(keep_lat);
    h->loaded = true;
    if ((h->flags & INFAAS_SEL_ENGINE_MASK) != INFAAS_SEL_ENGINE_SCAN) {
        int rc = create_index(h);
        if (rc != INFAAS_SEL_OK) {
            h->free_table();
            return rc;
        }
    }
    return INFAAS_SEL_OK;
}

int infaas_sel_update_load(infaas_sel_t *h, int32_t n, const int32_t *d_variant_idx,
                           const int32_t *d_queue_us, void *hip_stream)
{
    if (!h || n < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if (n == 0) return INFAAS_SEL_OK;
    if (!d_variant_idx || !d_queue_us) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        LaunchTimer t(h, INFAAS_SEL_K_UPDATE, st);
        if (!HIP_OK(launch_update_load(h->tv, n, d_variant_idx, d_queue_us,
                                       h->have_index ? &h->ix : nullptr, st, t.ev())))
            return INFAAS_SEL_ERR_HIP;
    }
    if (h->have_index) {  // the steps depend on the load: rebuild them behind the update
        h->steps_stale = true;
        LaunchTimer t(h, INFAAS_SEL_K_INDEX_BUILD, st);
        if (!HIP_OK(launch_index_build(h->tv, h->ix, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    return INFAAS_SEL_OK;
}

namespace {

// Gives the table of `h` the states (device copy of the caller's [V] array) and rebuilds its index.
int apply_states(infaas_sel *h, const int32_t *d_states, hipStream_t st)
{
    if (!HIP_OK(launch_update_state(h->tv, h->V, nullptr, d_states, h->have_index ? &h->ix : nullptr, st)))
        return INFAAS_SEL_ERR_HIP;
    h->steps_stale = true;
    if (h->have_index && !HIP_OK(launch_index_build(h->tv, h->ix, st))) return INFAAS_SEL_ERR_HIP;
    return INFAAS_SEL_OK;
}

}  // namespace

int infaas_sel_load_states(infaas_sel_t *h, const int32_t *state, const int32_t *load_us)
{
    if (!h) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if (!h->have_index || (h->V > 0 && (!state || !load_us))) return INFAAS_SEL_ERR_INVALID_ARG;
    const int32_t V = h->V, B = h->B;
    std::vector<int32_t> combined((size_t)V * B);   // load + inference latency: the Inactive tier's order
    for (int64_t v = 0; v < V; ++v) {
        if (state[v] < 0 || state[v] > 3 || load_us[v] < 0) return INFAAS_SEL_ERR_OUT_OF_RANGE;
        for (int32_t b = 0; b < B; ++b) {
            const int64_t c = (int64_t)load_us[v] + h->h_lat[(size_t)v * B + b];
            if (c > INT32_MAX) return INFAAS_SEL_ERR_OUT_OF_RANGE;
            combined[(size_t)v * B + b] = (int32_t)c;
        }
    }
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    h->drop_inactive();
    // The Inactive tier is a table of its own over the same rows: cost := load + latency (its order
    // is (load + latency, latency, row)) and queue := load (its latency test is load + latency <= slo).
    infaas_sel_config cfg{};
    cfg.num_tasks = h->T; cfg.num_batch_sizes = B; cfg.batch_sizes = h->batch_sizes.data();
    cfg.device = h->device; cfg.flags = INFAAS_SEL_ENGINE_INDEX; cfg.lds_segment_limit = h->lds_limit;
    infaas_sel *sub = nullptr;
    int rc = infaas_sel_create(&cfg, &sub);
    if (rc == INFAAS_SEL_OK)
        rc = infaas_sel_load_variants(sub, V, h->h_task.data(), h->h_acc.data(), h->h_lat.data(), combined.data(), load_us);
    if (rc == INFAAS_SEL_OK && !sub->have_index) rc = INFAAS_SEL_ERR_INVALID_ARG;
    int32_t *d_states = nullptr;
    if (rc == INFAAS_SEL_OK) {
        const size_t vp = (size_t)h->Vp;
        if (!h->d_state && dev_alloc(&h->d_state, vp) != hipSuccess) rc = INFAAS_SEL_ERR_OOM;
        if (rc == INFAAS_SEL_OK && dev_alloc(&sub->d_state, vp) != hipSuccess) rc = INFAAS_SEL_ERR_OOM;
        if (rc == INFAAS_SEL_OK && dev_alloc(&d_states, (size_t)std::max(V, 1)) != hipSuccess) rc = INFAAS_SEL_ERR_OOM;
        if (rc == INFAAS_SEL_ERR_OOM) (void)hipGetLastError();
    }
    if (rc == INFAAS_SEL_OK) {
        // padding slots get a state no table serves
        if (!HIP_OK(hipMemset(h->d_state, 0x7F, (size_t)h->Vp * 4)) || !HIP_OK(hipMemset(sub->d_state, 0x7F, (size_t)h->Vp * 4)) ||
            (V > 0 && !HIP_OK(hipMemcpy(d_states, state, (size_t)V * 4, hipMemcpyHostToDevice))))
            rc = INFAAS_SEL_ERR_HIP;
    }
    if (rc == INFAAS_SEL_OK) {
        h->tv.state = h->d_state; h->tv.want_state = 1;       // Active
        sub->tv.state = sub->d_state; sub->tv.want_state = 0; // Inactive
        rc = apply_states(h, d_states, nullptr);
        if (rc == INFAAS_SEL_OK) rc = apply_states(sub, d_states, nullptr);
        if (rc == INFAAS_SEL_OK && !HIP_OK(hipDeviceSynchronize())) rc = INFAAS_SEL_ERR_HIP;
    }
    (void)hipFree(d_states);
    if (rc != INFAAS_SEL_OK) {
        if (sub) infaas_sel_destroy(sub);
        // the states may have been applied to this table's columns already: rather than leave a
        // table that silently answers from some of its variants, drop it
        (void)hipDeviceSynchronize();
        h->free_table();
        return rc;
    }
    sub->timing = h->timing;
    h->inactive = sub;
    return INFAAS_SEL_OK;
}

int infaas_sel_update_state(infaas_sel_t *h, int32_t n, const int32_t *d_variant_idx,
                            const int32_t *d_state, void *hip_stream)
{
    if (!h || n < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->inactive) return INFAAS_SEL_ERR_NOT_LOADED;
    if (h->instance_states) return INFAAS_SEL_ERR_INVALID_ARG;   // a variant's state follows from its instances now
    if (n == 0) return INFAAS_SEL_OK;
    if (!d_variant_idx || !d_state) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    for (infaas_sel *t : {h, h->inactive}) {
        {
            LaunchTimer tm(t, INFAAS_SEL_K_UPDATE_STATE, st);
            if (!HIP_OK(launch_update_state(t->tv, n, d_variant_idx, d_state, &t->ix, st, tm.ev())))
                return INFAAS_SEL_ERR_HIP;
        }
        t->steps_stale = true;
        LaunchTimer tm(t, INFAAS_SEL_K_INDEX_BUILD, st);
        if (!HIP_OK(launch_index_build(t->tv, t->ix, st, tm.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    return INFAAS_SEL_OK;
}

namespace {

// Common part of the two select calls; d_out_closest is null for the plain one.
int select_impl(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                const int32_t *d_min_acc_bp, const int32_t *d_batch_idx, int32_t *d_out_variant,
                int32_t *d_out_closest, bool closest, void *hip_stream)
{
    if (!h || N < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if (closest && h->inactive) {
        snprintf(g_last_error, sizeof(g_last_error),
                 "infaas_sel_select_closest needs a handle without variant states (with states: infaas_sel_select_tiered_closest)");
        return INFAAS_SEL_ERR_INVALID_ARG;
    }
    if (N == 0) return INFAAS_SEL_OK;
    if (!d_task || !d_slo_us || !d_min_acc_bp || !d_batch_idx || !d_out_variant || (closest && !d_out_closest))
        return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    // (with variant states only the index honours them: its columns are masked, the scan's are not)
    // (the suggestion comes from the index whenever there is one; without one, from an exhaustive scan behind
    // the scan engine's selection)
    const bool idx = (closest && h->have_index) || h->inactive != nullptr || use_index(h);
    const bool groups = idx && !closest && !h->inactive && use_groups(h, std::min(N, kMaxPass));
    int rc = groups ? ensure_group_scratch(h, std::min(N, kMaxPass)) : idx ? INFAAS_SEL_OK : ensure_scratch(h, std::min(N, kMaxPass));
    if (rc != INFAAS_SEL_OK) return rc;
    for (int64_t done = 0; done < N; done += kMaxPass) {
        QueryView q{};
        q.n = (int32_t)std::min(kMaxPass, N - done);
        q.task = d_task + done; q.slo = d_slo_us + done; q.min_acc = d_min_acc_bp + done;
        q.bidx = d_batch_idx + done; q.out = d_out_variant + done;
        q.closest = closest ? d_out_closest + done : nullptr;
        q.pass = closest ? 1 : 0;
        rc = groups && q.n >= kGroupMinQueries ? group_pass(h, q, st) : idx ? index_pass(h, q, st) : scan_pass(h, q, st);
        if (rc != INFAAS_SEL_OK) return rc;
        if (closest && !idx) {
            LaunchTimer t(h, INFAAS_SEL_K_CLOSEST_SCAN, st);
            if (!HIP_OK(launch_closest_scan(h->tv, q, h->num_cus, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
        }
    }
    h->last_stats = idx ? h->ix.stats : nullptr;
    return INFAAS_SEL_OK;
}

}  // namespace

int infaas_sel_select(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                      const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                      int32_t *d_out_variant, void *hip_stream)
{
    return select_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, nullptr, false, hip_stream);
}

namespace {

// The state-aware selection, with the worker of every answer when d_out_worker is given and with
// the closest variant for the queries neither tier answers when d_out_closest is given.
int tiered_impl(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_worker, bool workers, void *hip_stream,
                int32_t *d_out_closest = nullptr, bool closest = false)
{
    if (!h || N < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->inactive || (workers && !h->workers_loaded)) return INFAAS_SEL_ERR_NOT_LOADED;
    if (N == 0) return INFAAS_SEL_OK;
    if (!d_task || !d_slo_us || !d_min_acc_bp || !d_batch_idx || !d_out_variant || !d_out_tier ||
        (workers && !d_out_worker) || (closest && !d_out_closest))
        return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = ensure_open(h, std::min(N, kMaxTierPass), closest);
    if (rc != INFAAS_SEL_OK) return rc;
    if (workers) {
        // bring the worker of every variant, then of every step of both indexes, up to date
        if (h->workers_dirty) {
            {
                LaunchTimer t(h, INFAAS_SEL_K_WORKER_TABLES, st);
                if (!HIP_OK(launch_best_per_class(h->wv, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
            }
            LaunchTimer t(h, INFAAS_SEL_K_WORKER_TABLES, st);
            if (!HIP_OK(launch_worker_tables(h->wv, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
            h->workers_dirty = false;
            h->steps_stale = h->inactive->steps_stale = true;
        }
        infaas_sel *tables[2] = {h, h->inactive};
        for (int tier = 0; tier < 2; ++tier) {
            infaas_sel *t = tables[tier];
            if (!t->steps_stale) continue;
            LaunchTimer tm(h, INFAAS_SEL_K_STEP_WORKERS, st);
            if (!HIP_OK(launch_step_workers(t->ix, h->wv.row_worker + (int64_t)tier * h->V, h->V, st, tm.ev())))
                return INFAAS_SEL_ERR_HIP;
            if (!HIP_OK(launch_hot_workers(t->ix, t->T * t->B, st))) return INFAAS_SEL_ERR_HIP;
            t->steps_stale = false;
        }
    }
    // The Active tier's lookup writes all result arrays and lists the valid queries it could not
    // answer; the Inactive tier's lookup reads only those lists and fills in what it can answer.
    for (int64_t done = 0; done < N; done += kMaxTierPass) {
        QueryView q{};
        q.n = (int32_t)std::min(kMaxTierPass, N - done);
        q.task = d_task + done; q.slo = d_slo_us + done; q.min_acc = d_min_acc_bp + done;
        q.bidx = d_batch_idx + done; q.out = d_out_variant + done; q.tier = d_out_tier + done;
        q.open = h->d_open; q.open_count = h->d_open_count;
        q.open_side = closest ? h->d_open + h->open_words : nullptr;
        q.open_cap = index_open_cap(q.n, h->num_cus);
        if (workers) { q.worker = d_out_worker + done; q.row_worker = h->wv.row_worker; }
        if (closest) q.closest = d_out_closest + done;
        q.pass = workers ? (closest ? 8 : 4) : closest ? 6 : 2;
        rc = index_pass(h, q, st);
        if (rc != INFAAS_SEL_OK) return rc;
        if (workers) q.row_worker = h->wv.row_worker + h->V;
        q.pass = workers ? (closest ? 9 : 5) : closest ? 7 : 3;
        rc = index_pass(h->inactive, q, st);
        if (rc != INFAAS_SEL_OK) return rc;
    }
    h->last_stats = h->inactive->ix.stats;
    return INFAAS_SEL_OK;
}

}  // namespace

int infaas_sel_select_tiered(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                             const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                             int32_t *d_out_variant, int32_t *d_out_tier, void *hip_stream)
{
    return tiered_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier, nullptr, false,
                       hip_stream);
}

int infaas_sel_select_tiered_closest(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                                     const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                                     int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_closest, void *hip_stream)
{
    return tiered_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier, nullptr, false,
                       hip_stream, d_out_closest, true);
}

int infaas_sel_select_workers(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_worker, void *hip_stream)
{
    return tiered_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier, d_out_worker, true,
                       hip_stream);
}

int infaas_sel_select_workers_closest(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                                      const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                                      int32_t *d_out_variant, int32_t *d_out_tier, int32_t *d_out_worker,
                                      int32_t *d_out_closest, void *hip_stream)
{
    return tiered_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier, d_out_worker, true,
                       hip_stream, d_out_closest, true);
}

int infaas_sel_load_workers(infaas_sel_t *h, int32_t num_workers, const int32_t *worker_hw, const int32_t *worker_util,
                            const int32_t *variant_hw, int32_t num_instances, const int32_t *inst_variant,
                            const int32_t *inst_worker, const int32_t *inst_load)
{
    if (!h || num_workers < 0 || num_instances < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->inactive) return INFAAS_SEL_ERR_NOT_LOADED;
    const int32_t V = h->V, W = num_workers, I = num_instances;
    if ((W > 0 && (!worker_hw || !worker_util)) || (V > 0 && !variant_hw) ||
        (I > 0 && (!inst_variant || !inst_worker || !inst_load)))
        return INFAAS_SEL_ERR_INVALID_ARG;
    for (int32_t w = 0; w < W; ++w)
        if (worker_util[w] < 0) return INFAAS_SEL_ERR_OUT_OF_RANGE;
    for (int32_t i = 0; i < I; ++i)
        if (inst_variant[i] < 0 || inst_variant[i] >= V || inst_worker[i] < 0 || inst_worker[i] >= W || inst_load[i] < 0)
            return INFAAS_SEL_ERR_OUT_OF_RANGE;
    // hardware classes that have workers, numbered in ascending order of the caller's codes
    std::vector<int32_t> codes(worker_hw, worker_hw + W);
    std::sort(codes.begin(), codes.end());
    codes.erase(std::unique(codes.begin(), codes.end()), codes.end());
    const int32_t H = (int32_t)codes.size();
    auto class_of = [&](int32_t code) -> int32_t {
        auto it = std::lower_bound(codes.begin(), codes.end(), code);
        return it != codes.end() && *it == code ? (int32_t)(it - codes.begin()) : -1;
    };
    std::vector<int32_t> cls_off((size_t)H + 1, 0), cls_worker((size_t)W), var_cls((size_t)V);
    for (int32_t w = 0; w < W; ++w) cls_off[(size_t)class_of(worker_hw[w]) + 1] += 1;
    for (int32_t c = 0; c < H; ++c) cls_off[(size_t)c + 1] += cls_off[(size_t)c];
    {
        std::vector<int32_t> at(cls_off.begin(), cls_off.end() - 1);
        for (int32_t w = 0; w < W; ++w) cls_worker[(size_t)at[(size_t)class_of(worker_hw[w])]++] = w;
    }
    for (int32_t v = 0; v < V; ++v) var_cls[(size_t)v] = class_of(variant_hw[v]);
    // instances grouped by variant
    std::vector<int32_t> inst_off((size_t)V + 1, 0), inst_w((size_t)I), inst_l((size_t)I), inst_pos((size_t)I);
    for (int32_t i = 0; i < I; ++i) inst_off[(size_t)inst_variant[i] + 1] += 1;
    for (int32_t v = 0; v < V; ++v) inst_off[(size_t)v + 1] += inst_off[(size_t)v];
    {
        std::vector<int32_t> at(inst_off.begin(), inst_off.end() - 1);
        for (int32_t i = 0; i < I; ++i) {
            const int32_t p = at[(size_t)inst_variant[i]]++;
            inst_w[(size_t)p] = inst_worker[i]; inst_l[(size_t)p] = inst_load[i]; inst_pos[(size_t)i] = p;
        }
    }
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    for (void *p : h->worker_mem) (void)hipFree(p);
    h->worker_mem.clear();
    h->workers_loaded = false;
    h->instance_states = false;
    bool ok = true;
    auto upload = [&](const std::vector<int32_t> &src, size_t count) -> int32_t * {
        int32_t *d = nullptr;
        if (!ok) return nullptr;
        if (dev_alloc(&d, count) != hipSuccess) { ok = false; (void)hipGetLastError(); return nullptr; }
        h->worker_mem.push_back(d);
        if (!src.empty() && !HIP_OK(hipMemcpy(d, src.data(), src.size() * 4, hipMemcpyHostToDevice))) ok = false;
        return d;
    };
    WorkerView wv{};
    wv.V = V; wv.W = W; wv.I = I; wv.H = H;
    wv.util = upload(std::vector<int32_t>(worker_util, worker_util + W), (size_t)W);
    wv.cls_off = upload(cls_off, cls_off.size());
    wv.cls_worker = upload(cls_worker, (size_t)W);
    wv.var_cls = upload(var_cls, (size_t)V);
    wv.inst_off = upload(inst_off, inst_off.size());
    wv.inst_worker = upload(inst_w, (size_t)I);
    wv.inst_load = upload(inst_l, (size_t)I);
    wv.inst_pos = upload(inst_pos, (size_t)I);
    wv.best_cls = upload({}, (size_t)H);
    wv.row_worker = upload({}, (size_t)2 * V);
    for (infaas_sel *t : {h, h->inactive}) {
        if (ok && !t->ix.step_worker && dev_alloc(&t->ix.step_worker, t->ix.step_cap) != hipSuccess) {
            ok = false;
            (void)hipGetLastError();
        }
        // 16-bit copies of the workers of the hot steps, for the lookup kernel's LDS
        (void)hipFree(t->ix.hot_worker);
        t->ix.hot_worker = nullptr;
        const size_t hot = (size_t)t->T * t->B * t->ix.hot_rows;
        if (ok && hot > 0 && t->index_lds_bytes > 0 && W <= 65535 &&
            dev_alloc(&t->ix.hot_worker, hot + 8) != hipSuccess) {
            ok = false;
            (void)hipGetLastError();
        }
        t->steps_stale = true;
    }
    if (!ok) {
        for (void *p : h->worker_mem) (void)hipFree(p);
        h->worker_mem.clear();
        h->wv = WorkerView{};
        return INFAAS_SEL_ERR_OOM;
    }
    h->wv = wv;
    h->workers_loaded = true;
    h->workers_dirty = true;
    return INFAAS_SEL_OK;
}

int infaas_sel_update_workers(infaas_sel_t *h, int32_t n, const int32_t *d_worker_idx, const int32_t *d_worker_util,
                              int32_t m, const int32_t *d_inst_idx, const int32_t *d_inst_load, void *hip_stream)
{
    if (!h || n < 0 || m < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->workers_loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if ((n > 0 && (!d_worker_idx || !d_worker_util)) || (m > 0 && (!d_inst_idx || !d_inst_load)))
        return INFAAS_SEL_ERR_INVALID_ARG;
    if (n == 0 && m == 0) return INFAAS_SEL_OK;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    LaunchTimer t(h, INFAAS_SEL_K_WORKER_REPORT, st);
    if (!HIP_OK(launch_worker_report(h->wv, n, d_worker_idx, d_worker_util, m, d_inst_idx, d_inst_load, st, t.ev())))
        return INFAAS_SEL_ERR_HIP;
    h->workers_dirty = true;
    return INFAAS_SEL_OK;
}

namespace {

// The variants' states derived anew from the instances', applied to both tiers' tables, both indexes
// rebuilt behind it (as after a state report).
int apply_instance_states(infaas_sel *h, hipStream_t st)
{
    {
        LaunchTimer t(h, INFAAS_SEL_K_INSTANCE_STATES, st);
        if (!HIP_OK(launch_derive_states(h->wv, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    for (infaas_sel *t : {h, h->inactive}) {
        {
            LaunchTimer tm(t, INFAAS_SEL_K_UPDATE_STATE, st);
            if (!HIP_OK(launch_update_state(t->tv, h->V, nullptr, h->wv.derived, &t->ix, st, tm.ev())))
                return INFAAS_SEL_ERR_HIP;
        }
        t->steps_stale = true;
        LaunchTimer tm(t, INFAAS_SEL_K_INDEX_BUILD, st);
        if (!HIP_OK(launch_index_build(t->tv, t->ix, st, tm.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    h->workers_dirty = true;
    return INFAAS_SEL_OK;
}

}  // namespace

int infaas_sel_load_instance_states(infaas_sel_t *h, const int32_t *inst_state)
{
    if (!h) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->inactive || !h->workers_loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    const int32_t I = h->wv.I;
    if (I > 0 && !inst_state) return INFAAS_SEL_ERR_INVALID_ARG;
    for (int32_t i = 0; i < I; ++i)
        if (inst_state[i] < INFAAS_SEL_STATE_ACTIVE || inst_state[i] > INFAAS_SEL_STATE_INTERFERED) return INFAAS_SEL_ERR_OUT_OF_RANGE;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    // in the order the instances are kept in: grouped by variant
    std::vector<int32_t> pos((size_t)I), grouped((size_t)I);
    if (I > 0 && !HIP_OK(hipMemcpy(pos.data(), h->wv.inst_pos, (size_t)I * 4, hipMemcpyDeviceToHost))) return INFAAS_SEL_ERR_HIP;
    for (int32_t i = 0; i < I; ++i) grouped[(size_t)pos[(size_t)i]] = inst_state[i];
    if (!h->wv.inst_state) {
        int32_t *d_st = nullptr, *d_der = nullptr;
        if (dev_alloc(&d_st, (size_t)std::max(I, 1)) != hipSuccess || dev_alloc(&d_der, (size_t)std::max(h->V, 1)) != hipSuccess) {
            (void)hipFree(d_st); (void)hipFree(d_der); (void)hipGetLastError();
            return INFAAS_SEL_ERR_OOM;
        }
        h->worker_mem.push_back(d_st); h->worker_mem.push_back(d_der);
        h->wv.inst_state = d_st; h->wv.derived = d_der;
    }
    if (I > 0 && !HIP_OK(hipMemcpy(h->wv.inst_state, grouped.data(), (size_t)I * 4, hipMemcpyHostToDevice))) return INFAAS_SEL_ERR_HIP;
    h->instance_states = true;
    int rc = apply_instance_states(h, nullptr);
    if (rc == INFAAS_SEL_OK && !HIP_OK(hipDeviceSynchronize())) rc = INFAAS_SEL_ERR_HIP;
    return rc;
}

int infaas_sel_update_instance_states(infaas_sel_t *h, int32_t n, const int32_t *d_inst_idx, const int32_t *d_state,
                                      void *hip_stream)
{
    if (!h || n < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->inactive || !h->workers_loaded || !h->instance_states) return INFAAS_SEL_ERR_NOT_LOADED;
    if (n == 0) return INFAAS_SEL_OK;
    if (!d_inst_idx || !d_state) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        LaunchTimer t(h, INFAAS_SEL_K_INSTANCE_STATES, st);
        if (!HIP_OK(launch_instance_state_report(h->wv, n, d_inst_idx, d_state, st, t.ev()))) return INFAAS_SEL_ERR_HIP;
    }
    return apply_instance_states(h, st);
}

int infaas_sel_select_noalloc(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, void *hip_stream)
{
    if (!h || N < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if (N > INFAAS_SEL_NOALLOC_MAX_QUERIES) {
        snprintf(g_last_error, sizeof(g_last_error), "infaas_sel_select_noalloc: %lld queries exceed the limit of %lld per call",
                 (long long)N, (long long)INFAAS_SEL_NOALLOC_MAX_QUERIES);
        return INFAAS_SEL_ERR_INVALID_ARG;
    }
    if (!h->have_index || !use_index(h)) {
        snprintf(g_last_error, sizeof(g_last_error),
                 "infaas_sel_select_noalloc needs the staircase index (the exhaustive scan buckets the queries in memory it allocates)");
        return INFAAS_SEL_ERR_INVALID_ARG;
    }
    if (index_park_bytes(h->num_cus) > kStaticScratchBytes) {
        snprintf(g_last_error, sizeof(g_last_error),
                 "infaas_sel_select_noalloc: the static scratch array is sized for %d compute units, this device has %d",
                 kStaticMaxCus, h->num_cus);
        return INFAAS_SEL_ERR_INVALID_ARG;
    }
    if (!h->static_park) {
        snprintf(g_last_error, sizeof(g_last_error), "infaas_sel_select_noalloc: the address of the static scratch array is not known");
        return INFAAS_SEL_ERR_HIP;
    }
    if (N == 0) return INFAAS_SEL_OK;
    if (!d_task || !d_slo_us || !d_min_acc_bp || !d_batch_idx || !d_out_variant) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    QueryView q{};
    q.n = (int32_t)N;
    q.task = d_task; q.slo = d_slo_us; q.min_acc = d_min_acc_bp; q.bidx = d_batch_idx; q.out = d_out_variant;
    q.pass = 0;
    // no event pair even when timing is on: taking one may create it
    if (!HIP_OK(launch_index_select(h->tv, h->ix, q, h->static_park, h->index_lds_bytes, h->num_cus,
                                    (hipStream_t)hip_stream, nullptr)))
        return INFAAS_SEL_ERR_HIP;
    h->last_stats = h->ix.stats;
    return INFAAS_SEL_OK;
}

int infaas_sel_select_closest(infaas_sel_t *h, int64_t N, const int32_t *d_task, const int32_t *d_slo_us,
                              const int32_t *d_min_acc_bp, const int32_t *d_batch_idx,
                              int32_t *d_out_variant, int32_t *d_out_closest, void *hip_stream)
{
    return select_impl(h, N, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_closest, true,
                       hip_stream);
}

int infaas_sel_load_scaling(infaas_sel_t *h, const int32_t *arch_id, const int32_t *sat_qps, const int32_t *hw_cost,
                            const int32_t *load_us, int32_t lambda_per_s, int32_t slack_pct)
{
    if (!h) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    const int32_t V = h->V, B = h->B;
    if (V > 0 && (!arch_id || !sat_qps || !hw_cost || !load_us)) return INFAAS_SEL_ERR_INVALID_ARG;
    if (lambda_per_s < 0 || lambda_per_s > 1000 || slack_pct < 0 || slack_pct > 200) return INFAAS_SEL_ERR_OUT_OF_RANGE;
    for (int32_t v = 0; v < V; ++v)
        if (sat_qps[v] < 1 || hw_cost[v] < 0 || hw_cost[v] > 1048576 || load_us[v] < 0) return INFAAS_SEL_ERR_OUT_OF_RANGE;
    // architectures numbered in ascending order of the caller's codes; their variants, rows ascending
    std::vector<int32_t> by_arch((size_t)V);
    std::iota(by_arch.begin(), by_arch.end(), 0);
    std::stable_sort(by_arch.begin(), by_arch.end(), [&](int32_t a, int32_t b) { return arch_id[a] < arch_id[b]; });
    std::vector<int32_t> arch_first;   // [A + 1] into by_arch
    for (int32_t p = 0; p < V; ++p)
        if (p == 0 || arch_id[by_arch[(size_t)p]] != arch_id[by_arch[(size_t)p - 1]]) arch_first.push_back(p);
    const int32_t A = (int32_t)arch_first.size();
    arch_first.push_back(V);
    auto unit_of = [&](int32_t v) {   // cost of one loaded instance, < 2^62
        return (uint64_t)hw_cost[v] * (1000000ull + (uint64_t)lambda_per_s * (uint64_t)load_us[v]);
    };
    // Candidates of an architecture at a batch size, for scaling up: by descending throughput, and only
    // those that no other variant beats for every request (at least the throughput, at most the latency,
    // and a lower cost per instance or the same with a lower row).  Sorted so that whatever beats a
    // variant comes before it; being beaten is transitive, so the survivors so far are enough to
    // compare with.  Every row of the architecture then gets its block: its own figures and the
    // first candidates of the prefix of the list whose throughput is above its own.
    // For scaling down: by ascending hardware cost, "beats" asks for at most the hardware cost besides
    // (a candidate must be cheaper than the running variant to be one at all), and a row's
    // candidates are the prefix of the list whose hardware cost is below its own.
    if ((int64_t)B * V * kScaleBlockWords * 4 > ((int64_t)1 << 33)) return INFAAS_SEL_ERR_OOM;   // 8 GB of blocks
    std::vector<uint32_t> blocks_of[2];
    std::vector<ScaleCand> cand_of[2];
    std::vector<int32_t> order, cand_cost;
    for (int down = 0; down < 2; ++down) {
        std::vector<uint32_t> &blocks = blocks_of[down];
        std::vector<ScaleCand> &cand = cand_of[down];
        blocks.assign((size_t)std::max<int64_t>((int64_t)B * V, 1) * kScaleBlockWords, 0u);
        if (V == 0) blocks[0] = 1u;   // the block an invalid request reads: throughput 1, no candidates (it is never used)
        cand_cost.clear();            // hardware cost of cand[k]
        for (int32_t b = 0; b < B; ++b)
            for (int32_t a = 0; a < A; ++a) {
                order.assign(by_arch.begin() + arch_first[(size_t)a], by_arch.begin() + arch_first[(size_t)a + 1]);
                std::sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
                    if (!down && sat_qps[x] != sat_qps[y]) return sat_qps[x] > sat_qps[y];
                    if (down && hw_cost[x] != hw_cost[y]) return hw_cost[x] < hw_cost[y];
                    const uint64_t ux = unit_of(x), uy = unit_of(y);
                    if (ux != uy) return ux < uy;
                    return x < y;
                });
                const size_t first = cand.size();
                for (int32_t v : order) {
                    const ScaleCand r{(uint32_t)sat_qps[v], h->h_lat[(size_t)v * B + b], unit_of(v), v, {0, 0, 0}};
                    bool beaten = false;
                    for (size_t k = first; k < cand.size() && !beaten; ++k)
                        beaten = cand[k].qps >= r.qps && cand[k].lat <= r.lat &&
                                 (cand[k].unit < r.unit || (cand[k].unit == r.unit && cand[k].row < v));
                    if (!beaten) { cand.push_back(r); cand_cost.push_back(hw_cost[v]); }
                }
                if (cand.size() > 0x7FFFFFFFull) return INFAAS_SEL_ERR_OUT_OF_RANGE;
                const size_t n = cand.size() - first;
                for (int32_t v : order) {
                    uint32_t *w = &blocks[((size_t)b * V + v) * kScaleBlockWords];
                    const uint64_t unit = unit_of(v);
                    size_t m = 0;   // candidates with a higher throughput, resp. a lower hardware cost: a prefix of the list
                    while (m < n && (down ? cand_cost[first + m] < hw_cost[v] : cand[first + m].qps > (uint32_t)sat_qps[v])) ++m;
                    w[0] = (uint32_t)sat_qps[v]; w[1] = (uint32_t)hw_cost[v];
                    w[2] = (uint32_t)unit; w[3] = (uint32_t)(unit >> 32);
                    w[4] = (uint32_t)h->h_lat[(size_t)v * B + b]; w[5] = (uint32_t)m; w[6] = (uint32_t)first;
                    for (size_t j = 0; j < std::min<size_t>(m, kScaleInBlock); ++j) {
                        const ScaleCand &c = cand[first + j];
                        uint32_t *sl = w + 8 + 4 * j;
                        sl[0] = c.qps; sl[1] = (uint32_t)c.lat; sl[2] = (uint32_t)c.unit; sl[3] = (uint32_t)(c.unit >> 32);
                        w[j < 4 ? 28 + j : 7] = (uint32_t)c.row;
                    }
                }
            }
        if (cand.empty()) cand.push_back(ScaleCand{1u, 0, 0ull, 0, {0, 0, 0}});
    }
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipDeviceSynchronize())) return INFAAS_SEL_ERR_HIP;
    for (void *p : h->scale_mem) (void)hipFree(p);
    h->scale_mem.clear();
    h->scaling_loaded = false;
    bool ok = true;
    auto upload = [&](const void *src, size_t bytes) -> void * {
        void *d = nullptr;
        if (!ok) return nullptr;
        if (hipMalloc(&d, std::max<size_t>(bytes, 16)) != hipSuccess) { ok = false; (void)hipGetLastError(); return nullptr; }
        h->scale_mem.push_back(d);
        if (bytes && !HIP_OK(hipMemcpy(d, src, bytes, hipMemcpyHostToDevice))) ok = false;
        return d;
    };
    ScaleView sv{};
    sv.V = V; sv.B = B; sv.slack_pct = slack_pct;
    sv.blocks = (const uint32_t *)upload(blocks_of[0].data(), blocks_of[0].size() * 4);
    sv.cand = (const ScaleCand *)upload(cand_of[0].data(), cand_of[0].size() * sizeof(ScaleCand));
    sv.blocks_down = (const uint32_t *)upload(blocks_of[1].data(), blocks_of[1].size() * 4);
    sv.cand_down = (const ScaleCand *)upload(cand_of[1].data(), cand_of[1].size() * sizeof(ScaleCand));
    if (!ok) {
        for (void *p : h->scale_mem) (void)hipFree(p);
        h->scale_mem.clear();
        return INFAAS_SEL_ERR_OOM;
    }
    h->sv = sv;
    h->scaling_loaded = true;
    return INFAAS_SEL_OK;
}

static int scale_impl(infaas_sel_t *h, bool down, int64_t R, const int32_t *d_variant, const int32_t *d_instances,
                      const int32_t *d_load_qps, const int32_t *d_slo_us, const int32_t *d_batch_idx,
                      int32_t *d_out_action, int32_t *d_out_variant, int32_t *d_out_instances, void *hip_stream)
{
    if (!h || R < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded || !h->scaling_loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    if (R == 0) return INFAAS_SEL_OK;
    if (!d_variant || !d_instances || !d_load_qps || !d_slo_us || !d_batch_idx || !d_out_action || !d_out_variant ||
        !d_out_instances)
        return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    LaunchTimer t(h, down ? INFAAS_SEL_K_SCALE_DOWN : INFAAS_SEL_K_SCALE, st);
    if (!HIP_OK(launch_scale(h->sv, down, R, d_variant, d_instances, d_load_qps, d_slo_us, d_batch_idx, d_out_action,
                             d_out_variant, d_out_instances, h->num_cus, st, t.ev())))
        return INFAAS_SEL_ERR_HIP;
    return INFAAS_SEL_OK;
}

int infaas_sel_scale(infaas_sel_t *h, int64_t R, const int32_t *d_variant, const int32_t *d_instances,
                     const int32_t *d_load_qps, const int32_t *d_slo_us, const int32_t *d_batch_idx,
                     int32_t *d_out_action, int32_t *d_out_variant, int32_t *d_out_instances, void *hip_stream)
{
    return scale_impl(h, false, R, d_variant, d_instances, d_load_qps, d_slo_us, d_batch_idx, d_out_action,
                      d_out_variant, d_out_instances, hip_stream);
}

int infaas_sel_scale_down(infaas_sel_t *h, int64_t R, const int32_t *d_variant, const int32_t *d_instances,
                          const int32_t *d_load_qps, const int32_t *d_slo_us, const int32_t *d_batch_idx,
                          int32_t *d_out_action, int32_t *d_out_variant, int32_t *d_out_instances, void *hip_stream)
{
    return scale_impl(h, true, R, d_variant, d_instances, d_load_qps, d_slo_us, d_batch_idx, d_out_action,
                      d_out_variant, d_out_instances, hip_stream);
}

void infaas_sel_destroy(infaas_sel_t *h)
{
    if (!h) return;
    {
        DeviceGuard g(h->device);
        (void)hipDeviceSynchronize();
        h->free_table();
        h->free_scratch();
        for (auto &p : h->pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        for (auto &e : h->free_events) (void)hipEventDestroy(e);
        if (h->host_stats) (void)hipHostFree(h->host_stats);
    }
    delete h;
}

int infaas_sel_reserve(infaas_sel_t *h, int64_t max_queries)
{
    if (!h || max_queries < 0) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    const int64_t cap = std::max<int64_t>(1, std::min(max_queries, kMaxPass));
    if (h->loaded && h->inactive) return ensure_open(h, std::min(cap, kMaxTierPass), h->open_side);
    if (h->loaded && use_index(h))   // the index engine needs per-query scratch only where it works group by group
        return use_groups(h, cap) ? ensure_group_scratch(h, cap) : INFAAS_SEL_OK;
    return ensure_scratch(h, cap);
}

int infaas_sel_read_load(infaas_sel_t *h, int32_t *queue_us, void *hip_stream)
{
    if (!h || !queue_us) return INFAAS_SEL_ERR_INVALID_ARG;
    if (!h->loaded) return INFAAS_SEL_ERR_NOT_LOADED;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    if (!HIP_OK(hipStreamSynchronize((hipStream_t)hip_stream))) return INFAAS_SEL_ERR_HIP;
    std::vector<int32_t> q(h->Vp), slot(std::max(h->V, 1));
    if (!HIP_OK(hipMemcpy(q.data(), h->d_queue, (size_t)h->Vp * 4, hipMemcpyDeviceToHost)) ||
        !HIP_OK(hipMemcpy(slot.data(), h->d_slot_of, (size_t)std::max(h->V, 1) * 4, hipMemcpyDeviceToHost)))
        return INFAAS_SEL_ERR_HIP;
    for (int32_t v = 0; v < h->V; ++v) queue_us[v] = q[slot[v]];
    return INFAAS_SEL_OK;
}

int infaas_sel_set_timing(infaas_sel_t *h, int32_t enabled)
{
    if (!h) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    for (auto &p : h->pending) {
        (void)hipEventSynchronize(p.b);
        h->free_events.push_back(p.a);
        h->free_events.push_back(p.b);
    }
    h->pending.clear();
    h->acc = infaas_sel_timings{};
    h->timing = enabled != 0;
    if (h->inactive) return infaas_sel_set_timing(h->inactive, enabled);
    return INFAAS_SEL_OK;
}

int infaas_sel_get_timings(infaas_sel_t *h, infaas_sel_timings *out)
{
    if (!h || !out) return INFAAS_SEL_ERR_INVALID_ARG;
    DeviceGuard g(h->device);
    if (!g.ok) return INFAAS_SEL_ERR_HIP;
    int rc = INFAAS_SEL_OK;
    for (auto &p : h->pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            h->acc.launches[p.kid] += 1;
            h->acc.total_ms[p.kid] += ms;
        } else {   // e.g. the launch itself failed and the events were never attached
            (void)hipGetLastError();
            rc = INFAAS_SEL_ERR_HIP;
        }
        h->free_events.push_back(p.a);
        h->free_events.push_back(p.b);
    }
    h->pending.clear();
    *out = h->acc;
    if (h->inactive) {   // the kernels of the Inactive tier's table count with this handle's
        infaas_sel_timings sub{};
        const int rc2 = infaas_sel_get_timings(h->inactive, &sub);
        for (int k = 0; k < INFAAS_SEL_K_COUNT; ++k) { out->launches[k] += sub.launches[k]; out->total_ms[k] += sub.total_ms[k]; }
        if (rc == INFAAS_SEL_OK) rc = rc2;
    }
    return rc;
}

int infaas_sel_get_info(infaas_sel_t *h, infaas_sel_info *out)
{
    if (!h || !out) return INFAAS_SEL_ERR_INVALID_ARG;
    std::memset(out, 0, sizeof(*out));
    out->num_variants = h->V;
    out->num_slices = h->T * h->B;
    out->max_segment = h->max_segment;
    out->lds_segment_limit = h->lds_limit;
    out->wide_segments = h->wide_segments;
    out->table_bytes = h->table_bytes;
    out->scratch_bytes = h->scratch_bytes + h->park_bytes + h->open_bytes + h->gs_bytes;
    if (h->have_index) {
        out->index_in_lds = h->index_lds_bytes > 0 ? 1 : 0;
        out->index_groups = (int32_t)h->ix.num_groups;
        // (as of the latest build that a selection has run behind, else as loaded)
        const volatile uint32_t *now = h->host_stats;
        out->index_truncated = (int32_t)(now ? now[kCtlTrunc - kCtlMaxK0] + now[kCtlNoBody - kCtlMaxK0]
                                             : h->ix_stats[kCtlTrunc] + h->ix_stats[kCtlNoBody]);
        out->index_max_steps = (int32_t)(now ? now[kCtlMaxK - kCtlMaxK0] : h->ix_stats[kCtlMaxK]);
        out->index_hot_rows = (int32_t)h->ix.hot_rows;
        // (with groups the two counters cover only what lies behind the regions: the figures of the load are kept)
        const bool fresh = now && h->ix.num_groups <= 1;
        const int64_t pool_now = fresh ? (int64_t)now[4] : h->ix_bytes, steps_now = fresh ? (int64_t)now[5] - 1 : h->ix_steps;
        out->index_bytes = pool_now + (int64_t)h->T * h->B * 16 + (steps_now + 1) * 4;
        out->index_steps = steps_now;
        // what the most recent lookup launch did with the queries its first probe could not decide
        std::vector<uint32_t> st((size_t)index_select_blocks(h->num_cus) * kLookupStats, 0u);
        DeviceGuard g(h->device);
        if (h->last_stats &&
            (!g.ok || !HIP_OK(hipMemcpy(st.data(), h->last_stats, st.size() * 4, hipMemcpyDeviceToHost)))) return INFAAS_SEL_ERR_HIP;
        int64_t sum[kLookupStats] = {0};
        for (size_t i = 0; i < st.size(); ++i) sum[i % kLookupStats] += st[i];
        out->lookup_parked = sum[0]; out->lookup_second_body = sum[1]; out->lookup_global_body = sum[2];
        out->lookup_scanned = sum[3]; out->lookup_unanswered = sum[4];
    }
    return INFAAS_SEL_OK;
}

}  // extern "C"
