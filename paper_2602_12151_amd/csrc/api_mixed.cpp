// C ABI of the mixed prefill + decode batch (declared in include/oserve.h): plan object and launch
// call.  Host code only; the kernel lives in mixed.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "host_util.h"
#include "kernels.h"
#include "oserve.h"
#include "plan.h"
#include "prefill_plan.h"

using oserve::PrefillItem;
using oserve::RunRecord;

namespace {

struct Layout {
    oserve::WorkspaceLayout decode;
    size_t queue_off, prefill_items_off, total;
};

}  // namespace

struct oserve_mixed_plan {
    oserve::SplitPlan decode;          // the requests that bring one query token
    oserve::PrefillWorkList prefill;   // the requests that bring more
    int32_t device_id = -1;
    int32_t compute_units = 256;       // the mixed kernel has two workgroups per compute unit
    std::vector<PrefillItem> items;    // prefill items as uploaded: XCD 0's queue, then XCD 1's, ...
    int32_t queue_first[oserve::kMaxXcds] = {}, queue_size[oserve::kMaxXcds] = {};
    // pinned staging ring: [run records][request info][prefill items] per slot
    char* staging = nullptr;
    char* staging_dev = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t upload_done[OSERVE_PLAN_RING] = {};
    bool slot_used[OSERVE_PLAN_RING] = {};
    int next_slot = 0;
    oserve::KernelTimer<OSERVE_PLAN_RING> timer;   // optional timing of the mixed kernel

    Layout layout(int64_t decode_items, int64_t row_groups, int32_t n, int64_t prefill_items) const {
        auto align = [](size_t x) { return (x + 255) & ~static_cast<size_t>(255); };
        Layout l{};
        l.decode = decode.layout(decode_items, row_groups, n);
        l.queue_off = l.decode.total;
        l.prefill_items_off = l.queue_off + align((oserve::kMaxQueueXcds + 1) * sizeof(int32_t));
        l.total = l.prefill_items_off + align(static_cast<size_t>(prefill_items) * sizeof(PrefillItem) + 16);
        return l;
    }
    Layout current_layout() const {
        return layout(decode.num_items, decode.num_row_groups, decode.batch, static_cast<int64_t>(items.size()));
    }
};

namespace {

using Guard = oserve::DeviceGuard;

void release(oserve_mixed_plan* pl) {
    for (int i = 0; i < OSERVE_PLAN_RING; ++i)
        if (pl->upload_done[i]) (void)hipEventDestroy(pl->upload_done[i]);
    pl->timer.destroy();
    if (pl->staging) (void)hipHostFree(pl->staging);
}

// Both work lists, then the launch order of the workgroups.
oserve_status_t build(oserve_mixed_plan* pl, const int32_t* lens, const int32_t* qlens, int32_t n) {
    if (!lens || !qlens) return OSERVE_ERR_NULL;
    // Everything the two builders check about the lengths is checked here first, so that a refused
    // update leaves both lists as they were.
    if (n < 1 || n > pl->prefill.capacity) return OSERVE_ERR_PLAN_MISMATCH;
    const int64_t max_len = static_cast<int64_t>(pl->prefill.geo.max_pages_per_seq) * pl->prefill.geo.page_size;
    int64_t total_q = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (lens[b] < 1 || lens[b] > max_len || qlens[b] < 1 || qlens[b] > lens[b]) return OSERVE_ERR_CONTEXT_LEN;
        total_q += qlens[b];
    }
    if (total_q > pl->prefill.max_query_tokens) return OSERVE_ERR_PLAN_MISMATCH;
    oserve_status_t st = pl->decode.build(lens, n, qlens);   // changes nothing unless it succeeds
    if (st != OSERVE_OK) return st;
    st = pl->prefill.build(lens, qlens, n, true);
    if (st != OSERVE_OK) return st;

    // prefill items as uploaded: the per-XCD lists one after the other, each a queue of the kernel
    // (inside a queue the blocks of one (request, kv head) follow each other, heaviest groups first)
    pl->items.clear();
    for (int x = 0; x < pl->prefill.xcds; ++x) {
        pl->queue_first[x] = static_cast<int32_t>(pl->items.size());
        pl->queue_size[x] = static_cast<int32_t>(pl->prefill.per_xcd[x].size());
        pl->items.insert(pl->items.end(), pl->prefill.per_xcd[x].begin(), pl->prefill.per_xcd[x].end());
    }
    return OSERVE_OK;
}

}  // namespace

extern "C" {

oserve_status_t oserve_mixed_plan_create(const int32_t* context_lens_host, const int32_t* q_lens_host,
                                         int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                         int32_t head_dim, int32_t page_size, int32_t max_pages_per_seq,
                                         int32_t device_id, int32_t capacity, int64_t max_query_tokens,
                                         oserve_mixed_plan_t** plan_out) {
    if (!plan_out) return OSERVE_ERR_NULL;
    *plan_out = nullptr;
    if (!context_lens_host || !q_lens_host) return OSERVE_ERR_NULL;
    const oserve::Geometry geo{num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq};
    oserve_status_t st = oserve::PrefillWorkList::check_geometry(geo, batch, capacity, max_query_tokens);
    if (st != OSERVE_OK) return st;
    if (device_id < -1) return OSERVE_ERR_SHAPE;

    oserve_mixed_plan* pl = new (std::nothrow) oserve_mixed_plan();
    if (!pl) return OSERVE_ERR_DEVICE;
    pl->device_id = device_id;
    pl->decode.geo = geo;
    pl->decode.capacity = capacity;
    pl->prefill.geo = geo;
    pl->prefill.capacity = capacity;
    pl->prefill.max_query_tokens = max_query_tokens;
    oserve::DeviceFacts facts;
    bool ok = true;
    if (device_id >= 0) {
        int n_dev = 0;
        ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev && oserve::query_device_facts(device_id, &facts);
        if (ok) {
            pl->decode.wave_slots = facts.compute_units * facts.simds_per_cu;
            pl->prefill.xcds = std::min<int32_t>(facts.xcds, oserve::kMaxXcds);
            pl->compute_units = facts.compute_units;
        }
    }
    if (!ok) { delete pl; return OSERVE_ERR_DEVICE; }
    pl->decode.reserve();
    pl->prefill.reserve();
    pl->items.reserve(static_cast<size_t>(pl->prefill.max_items()));
    pl->slot_bytes = (static_cast<size_t>(pl->decode.max_runs()) * sizeof(RunRecord) +
                      static_cast<size_t>(capacity) * sizeof(oserve::RequestInfo) +
                      static_cast<size_t>(pl->prefill.max_items()) * sizeof(PrefillItem) + 16 + 255) & ~static_cast<size_t>(255);
    if (device_id >= 0) {
        Guard guard(device_id);
        ok = guard.ok;
        ok = ok && hipHostMalloc(reinterpret_cast<void**>(&pl->staging), pl->slot_bytes * OSERVE_PLAN_RING,
                                 hipHostMallocDefault) == hipSuccess;
        ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&pl->staging_dev), pl->staging, 0) == hipSuccess;
        for (int i = 0; ok && i < OSERVE_PLAN_RING; ++i)
            ok = hipEventCreateWithFlags(&pl->upload_done[i], hipEventDisableTiming) == hipSuccess;
        ok = ok && pl->timer.create();
        if (!ok) { release(pl); delete pl; return OSERVE_ERR_DEVICE; }
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

oserve_status_t oserve_mixed_plan_update(oserve_mixed_plan_t* plan, const int32_t* context_lens_host,
                                         const int32_t* q_lens_host, int32_t batch) {
    if (!plan) return OSERVE_ERR_NULL;
    return build(plan, context_lens_host, q_lens_host, batch);
}

void oserve_mixed_plan_destroy(oserve_mixed_plan_t* plan) {
    if (!plan) return;
    if (plan->device_id >= 0) release(plan);
    delete plan;
}

int64_t oserve_mixed_plan_query_tokens(const oserve_mixed_plan_t* plan) { return plan->prefill.query_tokens; }

oserve_status_t oserve_mixed_plan_counts(const oserve_mixed_plan_t* plan, int32_t counts[4]) {
    if (!plan || !counts) return OSERVE_ERR_NULL;
    counts[0] = 2 * plan->compute_units;
    counts[1] = static_cast<int32_t>(plan->items.size());
    counts[2] = plan->decode.num_items;
    counts[3] = plan->prefill.xcds;
    return OSERVE_OK;
}

oserve_status_t oserve_mixed_plan_prefill_item(const oserve_mixed_plan_t* plan, int32_t i, int32_t fields[7]) {
    if (!plan || !fields) return OSERVE_ERR_NULL;
    if (i < 0 || i >= static_cast<int32_t>(plan->items.size())) return OSERVE_ERR_SHAPE;
    int32_t queue = 0;
    while (queue + 1 < plan->prefill.xcds && plan->queue_first[queue + 1] <= i) ++queue;
    fields[0] = queue;
    std::memcpy(fields + 1, &plan->items[i], 6 * sizeof(int32_t));
    return OSERVE_OK;
}

size_t oserve_mixed_plan_workspace_bytes(const oserve_mixed_plan_t* plan) { return plan->current_layout().total; }

size_t oserve_mixed_plan_workspace_bytes_max(const oserve_mixed_plan_t* plan) {
    const int64_t items = plan->decode.max_items();
    return plan->layout(items, items / plan->decode.geo.num_kv_heads, plan->decode.capacity, plan->prefill.max_items()).total;
}

oserve_status_t oserve_paged_mixed_attn(oserve_mixed_plan_t* plan, void* workspace, size_t workspace_bytes,
                                        const void* q, const void* k_pages, const void* v_pages,
                                        const int32_t* block_table, const int32_t* context_lens, float scale,
                                        float* out, void* stream_v) {
    if (!plan || !workspace || !q || !k_pages || !v_pages || !block_table || !context_lens || !out)
        return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    if (!(scale > 0.f) || !std::isfinite(scale)) return OSERVE_ERR_SHAPE;   // the prefill side orders raw scores
    const oserve::SplitPlan& dp = plan->decode;
    const Layout lay = plan->current_layout();
    if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return OSERVE_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pages) |
         reinterpret_cast<uintptr_t>(v_pages) | reinterpret_cast<uintptr_t>(out)) & 15u)
        return OSERVE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    Guard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;

    const int slot = plan->next_slot;
    plan->next_slot = (slot + 1) % OSERVE_PLAN_RING;
    if (plan->slot_used[slot] && hipEventSynchronize(plan->upload_done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    if (plan->timer.enabled && !plan->timer.collect(slot)) return OSERVE_ERR_DEVICE;
    // slot: [run records][request info][prefill items], each part a multiple of 16 bytes
    const size_t slot_off = static_cast<size_t>(slot) * plan->slot_bytes;
    const size_t n_runs = dp.records.size();
    const size_t info_off = sizeof(RunRecord) * n_runs;
    const size_t items_off = info_off + sizeof(oserve::RequestInfo) * static_cast<size_t>(dp.batch);
    const size_t items_bytes = plan->items.size() * sizeof(PrefillItem);
    char* st_host = plan->staging + slot_off;
    std::memcpy(st_host, dp.records.data(), info_off);
    std::memcpy(st_host + info_off, dp.req_info.data(), items_off - info_off);
    std::memcpy(st_host + items_off, plan->items.data(), items_bytes);

    char* ws = static_cast<char*>(workspace);
    const char* st_dev = plan->staging_dev + slot_off;
    oserve::ExpandParams ep{};
    ep.records_host = reinterpret_cast<const RunRecord*>(st_dev);
    ep.num_runs = static_cast<int32_t>(n_runs);
    ep.req_info_host = reinterpret_cast<const oserve::RequestInfo*>(st_dev + info_off);
    ep.req_info = reinterpret_cast<oserve::RequestInfo*>(ws + lay.decode.req_info_off);
    ep.batch = dp.batch;
    ep.items = reinterpret_cast<oserve::ItemDesc*>(ws + lay.decode.items_off);
    ep.num_kv_heads = dp.geo.num_kv_heads;
    ep.kv_heads_magic = static_cast<uint32_t>((1ull << 32) / static_cast<uint32_t>(dp.geo.num_kv_heads)) + 1u;
    ep.blob_host = st_dev + items_off;
    ep.blob = ws + lay.prefill_items_off;
    ep.blob_words = static_cast<int32_t>(items_bytes / 16);
    ep.zero = reinterpret_cast<int32_t*>(ws + lay.queue_off);
    ep.zero_words = oserve::kMaxQueueXcds + 1;
    if (oserve::launch_expand(ep, stream, plan->upload_done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    plan->slot_used[slot] = true;

    const int32_t tile_shift = dp.geo.page_size == 64 ? 2 : dp.geo.page_size == 32 ? 1 : 0;
    oserve::MixedParams mp{};
    oserve::SplitParams& sp = mp.decode;
    sp.items = ep.items;
    sp.req_info = ep.req_info;
    sp.q = static_cast<const uint16_t*>(q);
    sp.k_pages = static_cast<const uint16_t*>(k_pages);
    sp.v_pages = static_cast<const uint16_t*>(v_pages);
    sp.block_table = block_table;
    sp.context_lens = context_lens;
    sp.out = out;
    sp.partial_o = reinterpret_cast<float*>(ws + lay.decode.partial_o_off);
    sp.partial_ml = reinterpret_cast<float*>(ws + lay.decode.partial_ml_off);
    sp.scale_log2e = scale * 1.44269504088896340736f;
    sp.num_q_heads = dp.geo.num_q_heads;
    sp.num_kv_heads = dp.geo.num_kv_heads;
    sp.group = dp.geo.group();
    sp.max_pages_per_seq = dp.geo.max_pages_per_seq;
    sp.tile_shift = tile_shift;
    oserve::PrefillParams& pp = mp.prefill;
    pp.items = reinterpret_cast<const PrefillItem*>(ws + lay.prefill_items_off);
    pp.q = sp.q;
    pp.k_pages = sp.k_pages;
    pp.v_pages = sp.v_pages;
    pp.block_table = block_table;
    pp.out = out;
    pp.scale_log2e = sp.scale_log2e;
    pp.num_q_heads = sp.num_q_heads;
    pp.num_kv_heads = sp.num_kv_heads;
    pp.group = sp.group;
    pp.group_shift = plan->prefill.group_shift();
    pp.max_pages_per_seq = sp.max_pages_per_seq;
    pp.tile_shift = tile_shift;
    mp.queue_next = ep.zero;
    for (int x = 0; x < oserve::kMaxQueueXcds; ++x) {
        mp.prefill_queue_first[x] = x < plan->prefill.xcds ? plan->queue_first[x] : 0;
        mp.prefill_queue_size[x] = x < plan->prefill.xcds ? plan->queue_size[x] : 0;
    }
    mp.num_xcds = plan->prefill.xcds;
    mp.num_decode_items = dp.num_items;
    if (oserve::launch_mixed(mp, dp.geo.head_dim, 2 * plan->compute_units, stream,
                             plan->timer.begin_of(slot), plan->timer.end_of(slot)) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    plan->timer.mark(slot);

    if (dp.needs_merge) {
        oserve::MergeParams gp{};
        gp.req_info = ep.req_info;
        gp.partial_o = sp.partial_o;
        gp.partial_ml = sp.partial_ml;
        gp.out = out;
        gp.num_q_heads = sp.num_q_heads;
        if (oserve::launch_merge(gp, dp.geo.head_dim, dp.batch, stream) != hipSuccess) return OSERVE_ERR_DEVICE;
    }
    return OSERVE_OK;
}

oserve_status_t oserve_mixed_plan_enable_timing(oserve_mixed_plan_t* plan, int32_t enable) {
    if (!plan) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.set_enabled(enable != 0) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

oserve_status_t oserve_mixed_plan_kernel_ms(oserve_mixed_plan_t* plan, float* mean_ms, int32_t* count) {
    if (!plan || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.mean(mean_ms, count) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

}  // extern "C"
