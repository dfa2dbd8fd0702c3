// C ABI of the chunked-prefill path (declared in include/oserve.h): plan objects and the launch
// call.  Host code only; the kernel lives in prefill.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.h"
#include "oserve.h"
#include "plan.h"

using oserve::PrefillItem;

struct oserve_prefill_plan {
    oserve::Geometry geo{};
    int32_t capacity = 0;            // largest batch
    int64_t max_query_tokens = 0;    // largest sum of query lengths
    int32_t device_id = -1;
    int32_t batch = 0;
    int64_t query_tokens = 0;
    static constexpr int kXcds = 8;  // accelerator dies of the device, each with its own L2
    std::vector<PrefillItem> items;  // launch order
    std::vector<PrefillItem> scratch;
    std::vector<PrefillItem> per_xcd[kXcds];
    struct Group { int32_t request, kv_head; int64_t work; };
    std::vector<Group> groups;
    std::vector<int64_t> row0;
    // ring of pinned staging slots read directly by the kernel; `done` completes with the kernel
    char* staging = nullptr;
    char* staging_dev = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t done[OSERVE_PLAN_RING] = {};
    bool slot_used[OSERVE_PLAN_RING] = {};
    int next_slot = 0;
    // optional kernel timing
    bool timing = false;
    hipEvent_t t_begin[OSERVE_PLAN_RING] = {}, t_end[OSERVE_PLAN_RING] = {};
    bool t_pending[OSERVE_PLAN_RING] = {};
    double t_sum_ms = 0.0;
    int64_t t_count = 0;

    int32_t group_shift() const {
        int32_t s = 0;
        while ((1 << s) < geo.group()) ++s;
        return s;
    }
    int32_t block_tokens() const { return oserve::prefill_block_tokens(group_shift()); }   // query tokens per workgroup
    int64_t max_items() const {
        return (max_query_tokens / block_tokens() + capacity) * geo.num_kv_heads;
    }
};

namespace {

struct Guard {
    int prev = -1, target = -1;
    bool ok = true;
    explicit Guard(int dev) : target(dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~Guard() { if (ok && prev != target) (void)hipSetDevice(prev); }
};

void release(oserve_prefill_plan* pl) {
    for (int i = 0; i < OSERVE_PLAN_RING; ++i) {
        if (pl->done[i]) (void)hipEventDestroy(pl->done[i]);
        if (pl->t_begin[i]) (void)hipEventDestroy(pl->t_begin[i]);
        if (pl->t_end[i]) (void)hipEventDestroy(pl->t_end[i]);
    }
    if (pl->staging) (void)hipHostFree(pl->staging);
}

bool collect(oserve_prefill_plan* pl, int slot) {
    if (!pl->t_pending[slot]) return true;
    if (hipEventSynchronize(pl->t_end[slot]) != hipSuccess) return false;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, pl->t_begin[slot], pl->t_end[slot]) != hipSuccess) return false;
    pl->t_sum_ms += ms;
    pl->t_count += 1;
    pl->t_pending[slot] = false;
    return true;
}

// Work items: blocks of query tokens x kv heads, ordered for L2 reuse and balance (see below).
oserve_status_t build(oserve_prefill_plan* pl, const int32_t* lens, const int32_t* qlens, int32_t n) {
    if (!lens || !qlens) return OSERVE_ERR_NULL;
    if (n < 1 || n > pl->capacity) return OSERVE_ERR_PLAN_MISMATCH;
    const int64_t max_len = static_cast<int64_t>(pl->geo.max_pages_per_seq) * pl->geo.page_size;
    int64_t total_q = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (lens[b] < 1 || lens[b] > max_len || qlens[b] < 1 || qlens[b] > lens[b]) return OSERVE_ERR_CONTEXT_LEN;
        total_q += qlens[b];
    }
    if (total_q > pl->max_query_tokens) return OSERVE_ERR_PLAN_MISMATCH;
    const int32_t qb = pl->block_tokens();
    const int32_t hkv = pl->geo.num_kv_heads;
    // Groups = (request, kv head): all query blocks of a group read the same K/V.  Workgroups go to
    // the device's XCDs round-robin by index, and every XCD has its own L2, so the blocks of a group
    // are placed at indices that are equal modulo the XCD count: they then run side by side on one
    // XCD and its L2 serves the K/V tiles that the first of them fetched.  Groups are dealt to the
    // XCDs heaviest first, each to the XCD with the least work so far; inside a group the blocks
    // with the most keys come first.
    using Group = oserve_prefill_plan::Group;
    std::vector<Group>& groups = pl->groups;
    groups.clear();
    for (int32_t b = 0; b < n; ++b) {
        int64_t work = 0;
        for (int32_t q0 = 0; q0 < qlens[b]; q0 += qb)
            work += lens[b] - qlens[b] + std::min(q0 + qb, qlens[b]);
        for (int32_t j = 0; j < hkv; ++j) groups.push_back(Group{b, j, work});
    }
    std::stable_sort(groups.begin(), groups.end(), [](const Group& a, const Group& c) { return a.work > c.work; });
    std::vector<int64_t>& row0 = pl->row0;
    row0.assign(static_cast<size_t>(n) + 1, 0);
    for (int32_t b = 0; b < n; ++b) row0[b + 1] = row0[b] + qlens[b];
    constexpr int kXcds = oserve_prefill_plan::kXcds;
    int64_t load[kXcds] = {};
    for (int x = 0; x < kXcds; ++x) pl->per_xcd[x].clear();
    for (const Group& g : groups) {
        int best = 0;
        for (int x = 1; x < kXcds; ++x)
            if (load[x] < load[best]) best = x;
        load[best] += g.work;
        const int32_t b = g.request;
        const int32_t blocks = (qlens[b] + qb - 1) / qb;
        for (int32_t k = blocks - 1; k >= 0; --k)     // last blocks see the most keys
            pl->per_xcd[best].push_back(PrefillItem{b, g.kv_head, k * qb, static_cast<int32_t>(row0[b]), lens[b], qlens[b], {0, 0}});
    }
    // interleave: position 8 k + x takes the k-th item of XCD x's list; exhausted lists are skipped
    std::vector<PrefillItem>& it = pl->scratch;
    it.clear();
    size_t cursor[kXcds] = {};
    for (bool any = true; any;) {
        any = false;
        for (int x = 0; x < kXcds; ++x)
            if (cursor[x] < pl->per_xcd[x].size()) {
                it.push_back(pl->per_xcd[x][cursor[x]++]);
                any = true;
            }
    }
    pl->items.swap(it);
    pl->batch = n;
    pl->query_tokens = total_q;
    return OSERVE_OK;
}

}  // namespace

extern "C" {

oserve_status_t oserve_prefill_plan_create(const int32_t* context_lens_host, const int32_t* q_lens_host,
                                           int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                           int32_t head_dim, int32_t page_size, int32_t max_pages_per_seq,
                                           int32_t device_id, int32_t capacity, int64_t max_query_tokens,
                                           oserve_prefill_plan_t** plan_out) {
    if (!plan_out) return OSERVE_ERR_NULL;
    *plan_out = nullptr;
    if (!context_lens_host || !q_lens_host) return OSERVE_ERR_NULL;
    const oserve::Geometry geo{num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq};
    oserve_status_t st = oserve::SplitPlan::check_geometry(geo, batch, capacity, 0);
    if (st != OSERVE_OK) return st;
    const int32_t g = geo.group();
    if (head_dim != 128 || (g & (g - 1)) != 0) return OSERVE_ERR_SHAPE;   // group 1, 2, 4, 8 or 16
    if (device_id < -1 || max_query_tokens < 1 || max_query_tokens > (1ll << 28)) return OSERVE_ERR_SHAPE;

    oserve_prefill_plan* pl = new (std::nothrow) oserve_prefill_plan();
    if (!pl) return OSERVE_ERR_DEVICE;
    pl->geo = geo;
    pl->capacity = capacity;
    pl->max_query_tokens = max_query_tokens;
    pl->device_id = device_id;
    pl->items.reserve(static_cast<size_t>(pl->max_items()));
    pl->scratch.reserve(static_cast<size_t>(pl->max_items()));
    for (auto& v : pl->per_xcd) v.reserve(static_cast<size_t>(pl->max_items()));
    pl->groups.reserve(static_cast<size_t>(capacity) * num_kv_heads);
    pl->row0.reserve(static_cast<size_t>(capacity) + 1);
    pl->slot_bytes = (static_cast<size_t>(pl->max_items()) * sizeof(PrefillItem) + 255) & ~static_cast<size_t>(255);
    if (device_id >= 0) {
        int n_dev = 0;
        bool ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev;
        if (ok) {
            Guard guard(device_id);
            ok = guard.ok;
            ok = ok && hipHostMalloc(reinterpret_cast<void**>(&pl->staging), pl->slot_bytes * OSERVE_PLAN_RING,
                                     hipHostMallocDefault) == hipSuccess;
            ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&pl->staging_dev), pl->staging, 0) == hipSuccess;
            for (int i = 0; ok && i < OSERVE_PLAN_RING; ++i) {
                ok = hipEventCreateWithFlags(&pl->done[i], hipEventDisableTiming) == hipSuccess;
                ok = ok && hipEventCreate(&pl->t_begin[i]) == hipSuccess;
                ok = ok && hipEventCreate(&pl->t_end[i]) == hipSuccess;
            }
        }
        if (!ok) {
            release(pl);
            delete pl;
            return OSERVE_ERR_DEVICE;
        }
    }
    st = build(pl, context_lens_host, q_lens_host, batch);
    if (st != OSERVE_OK) {
        if (device_id >= 0) release(pl);
        delete pl;
        return st;
    }
    *plan_out = pl;
    return OSERVE_OK;
}

oserve_status_t oserve_prefill_plan_update(oserve_prefill_plan_t* plan, const int32_t* context_lens_host,
                                           const int32_t* q_lens_host, int32_t batch) {
    if (!plan) return OSERVE_ERR_NULL;
    return build(plan, context_lens_host, q_lens_host, batch);
}

void oserve_prefill_plan_destroy(oserve_prefill_plan_t* plan) {
    if (!plan) return;
    if (plan->device_id >= 0) release(plan);
    delete plan;
}

int32_t oserve_prefill_plan_num_work_items(const oserve_prefill_plan_t* plan) {
    return static_cast<int32_t>(plan->items.size());
}
int64_t oserve_prefill_plan_query_tokens(const oserve_prefill_plan_t* plan) { return plan->query_tokens; }
int32_t oserve_prefill_plan_block_tokens(const oserve_prefill_plan_t* plan) { return plan->block_tokens(); }

oserve_status_t oserve_prefill_plan_item(const oserve_prefill_plan_t* plan, int32_t i, int32_t fields[6]) {
    if (!plan || !fields) return OSERVE_ERR_NULL;
    if (i < 0 || i >= static_cast<int32_t>(plan->items.size())) return OSERVE_ERR_SHAPE;
    std::memcpy(fields, &plan->items[i], 6 * sizeof(int32_t));
    return OSERVE_OK;
}

oserve_status_t oserve_paged_prefill_attn(oserve_prefill_plan_t* plan, const void* q, const void* k_pages,
                                          const void* v_pages, const int32_t* block_table, float scale,
                                          float* out, void* stream_v) {
    if (!plan || !q || !k_pages || !v_pages || !block_table || !out) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    if (!(scale > 0.f) || !std::isfinite(scale)) return OSERVE_ERR_SHAPE;   // the kernel orders raw scores
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pages) |
         reinterpret_cast<uintptr_t>(v_pages) | reinterpret_cast<uintptr_t>(out)) & 15u)
        return OSERVE_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    Guard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;

    const int slot = plan->next_slot;
    plan->next_slot = (slot + 1) % OSERVE_PLAN_RING;
    if (plan->slot_used[slot] && hipEventSynchronize(plan->done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    if (plan->timing && !collect(plan, slot)) return OSERVE_ERR_DEVICE;
    const size_t off = static_cast<size_t>(slot) * plan->slot_bytes;
    std::memcpy(plan->staging + off, plan->items.data(), plan->items.size() * sizeof(PrefillItem));

    oserve::PrefillParams pp{};
    pp.items = reinterpret_cast<const PrefillItem*>(plan->staging_dev + off);
    pp.q = static_cast<const uint16_t*>(q);
    pp.k_pages = static_cast<const uint16_t*>(k_pages);
    pp.v_pages = static_cast<const uint16_t*>(v_pages);
    pp.block_table = block_table;
    pp.out = out;
    pp.scale_log2e = scale * 1.44269504088896340736f;
    pp.num_q_heads = plan->geo.num_q_heads;
    pp.num_kv_heads = plan->geo.num_kv_heads;
    pp.group = plan->geo.group();
    pp.group_shift = plan->group_shift();
    pp.max_pages_per_seq = plan->geo.max_pages_per_seq;
    pp.tile_shift = plan->geo.page_size == 64 ? 2 : plan->geo.page_size == 32 ? 1 : 0;
    const int n_items = static_cast<int>(plan->items.size());
    if (plan->timing) {
        if (oserve::launch_prefill(pp, plan->geo.head_dim, n_items, stream, plan->t_begin[slot], plan->t_end[slot]) != hipSuccess)
            return OSERVE_ERR_DEVICE;
        plan->t_pending[slot] = true;
        if (hipEventRecord(plan->done[slot], stream) != hipSuccess) return OSERVE_ERR_DEVICE;
    } else if (oserve::launch_prefill(pp, plan->geo.head_dim, n_items, stream, nullptr, plan->done[slot]) != hipSuccess) {
        return OSERVE_ERR_DEVICE;
    }
    plan->slot_used[slot] = true;
    return OSERVE_OK;
}

oserve_status_t oserve_prefill_plan_enable_timing(oserve_prefill_plan_t* plan, int32_t enable) {
    if (!plan) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    for (int i = 0; i < OSERVE_PLAN_RING; ++i)
        if (!collect(plan, i)) return OSERVE_ERR_DEVICE;
    plan->timing = enable != 0;
    plan->t_sum_ms = 0.0;
    plan->t_count = 0;
    return OSERVE_OK;
}

oserve_status_t oserve_prefill_plan_kernel_ms(oserve_prefill_plan_t* plan, float* mean_ms, int32_t* count) {
    if (!plan || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    for (int i = 0; i < OSERVE_PLAN_RING; ++i)
        if (!collect(plan, i)) return OSERVE_ERR_DEVICE;
    *count = static_cast<int32_t>(plan->t_count);
    *mean_ms = plan->t_count ? static_cast<float>(plan->t_sum_ms / plan->t_count) : 0.f;
    return OSERVE_OK;
}

}  // extern "C"
