// C ABI of the chunked-prefill path (declared in include/oserve.h): plan objects and the launch
// call.  Host code only; the kernel lives in prefill.hip.
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

struct oserve_prefill_plan {
    oserve::PrefillWorkList list;
    int32_t device_id = -1;
    // ring of pinned staging slots read directly by the kernel; `done` completes with the kernel
    char* staging = nullptr;
    char* staging_dev = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t done[OSERVE_PLAN_RING] = {};
    bool slot_used[OSERVE_PLAN_RING] = {};
    int next_slot = 0;
    oserve::KernelTimer<OSERVE_PLAN_RING> timer;   // optional kernel timing
};

namespace {

using Guard = oserve::DeviceGuard;

void release(oserve_prefill_plan* pl) {
    for (int i = 0; i < OSERVE_PLAN_RING; ++i) {
        if (pl->done[i]) (void)hipEventDestroy(pl->done[i]);
    }
    pl->timer.destroy();
    if (pl->staging) (void)hipHostFree(pl->staging);
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
    oserve_status_t st = oserve::PrefillWorkList::check_geometry(geo, batch, capacity, max_query_tokens);
    if (st != OSERVE_OK) return st;
    if (device_id < -1) return OSERVE_ERR_SHAPE;

    oserve_prefill_plan* pl = new (std::nothrow) oserve_prefill_plan();
    if (!pl) return OSERVE_ERR_DEVICE;
    pl->list.geo = geo;
    pl->list.capacity = capacity;
    pl->list.max_query_tokens = max_query_tokens;
    pl->device_id = device_id;
    pl->slot_bytes = (static_cast<size_t>(pl->list.max_items()) * sizeof(PrefillItem) + 255) & ~static_cast<size_t>(255);
    if (device_id >= 0) {
        int n_dev = 0;
        oserve::DeviceFacts facts;
        bool ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev;
        ok = ok && oserve::query_device_facts(device_id, &facts);
        if (ok) {
            pl->list.xcds = std::min<int32_t>(facts.xcds, oserve::kMaxXcds);
            Guard guard(device_id);
            ok = guard.ok;
            ok = ok && hipHostMalloc(reinterpret_cast<void**>(&pl->staging), pl->slot_bytes * OSERVE_PLAN_RING,
                                     hipHostMallocDefault) == hipSuccess;
            ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&pl->staging_dev), pl->staging, 0) == hipSuccess;
            for (int i = 0; ok && i < OSERVE_PLAN_RING; ++i) {
                ok = hipEventCreateWithFlags(&pl->done[i], hipEventDisableTiming) == hipSuccess;
            }
            ok = ok && pl->timer.create();
        }
        if (!ok) {
            release(pl);
            delete pl;
            return OSERVE_ERR_DEVICE;
        }
    }
    pl->list.reserve();
    st = pl->list.build(context_lens_host, q_lens_host, batch, false);
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
    return plan->list.build(context_lens_host, q_lens_host, batch, false);
}

void oserve_prefill_plan_destroy(oserve_prefill_plan_t* plan) {
    if (!plan) return;
    if (plan->device_id >= 0) release(plan);
    delete plan;
}

int32_t oserve_prefill_plan_num_work_items(const oserve_prefill_plan_t* plan) {
    return static_cast<int32_t>(plan->list.items.size());
}
int64_t oserve_prefill_plan_query_tokens(const oserve_prefill_plan_t* plan) { return plan->list.query_tokens; }
int32_t oserve_prefill_plan_block_tokens(const oserve_prefill_plan_t* plan) { return plan->list.block_tokens(); }

oserve_status_t oserve_prefill_plan_item(const oserve_prefill_plan_t* plan, int32_t i, int32_t fields[6]) {
    if (!plan || !fields) return OSERVE_ERR_NULL;
    if (i < 0 || i >= static_cast<int32_t>(plan->list.items.size())) return OSERVE_ERR_SHAPE;
    std::memcpy(fields, &plan->list.items[i], 6 * sizeof(int32_t));
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
        return OSERVE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    Guard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;

    const int slot = plan->next_slot;
    plan->next_slot = (slot + 1) % OSERVE_PLAN_RING;
    if (plan->slot_used[slot] && hipEventSynchronize(plan->done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    if (plan->timer.enabled && !plan->timer.collect(slot)) return OSERVE_ERR_DEVICE;
    const size_t off = static_cast<size_t>(slot) * plan->slot_bytes;
    std::memcpy(plan->staging + off, plan->list.items.data(), plan->list.items.size() * sizeof(PrefillItem));

    oserve::PrefillParams pp{};
    pp.items = reinterpret_cast<const PrefillItem*>(plan->staging_dev + off);
    pp.q = static_cast<const uint16_t*>(q);
    pp.k_pages = static_cast<const uint16_t*>(k_pages);
    pp.v_pages = static_cast<const uint16_t*>(v_pages);
    pp.block_table = block_table;
    pp.out = out;
    pp.scale_log2e = scale * 1.44269504088896340736f;
    pp.num_q_heads = plan->list.geo.num_q_heads;
    pp.num_kv_heads = plan->list.geo.num_kv_heads;
    pp.group = plan->list.geo.group();
    pp.group_shift = plan->list.group_shift();
    pp.max_pages_per_seq = plan->list.geo.max_pages_per_seq;
    pp.tile_shift = plan->list.geo.page_size == 64 ? 2 : plan->list.geo.page_size == 32 ? 1 : 0;
    const int n_items = static_cast<int>(plan->list.items.size());
    if (plan->timer.enabled) {
        if (oserve::launch_prefill(pp, plan->list.geo.head_dim, n_items, stream, plan->timer.begin_of(slot), plan->timer.end_of(slot)) != hipSuccess)
            return OSERVE_ERR_DEVICE;
        plan->timer.mark(slot);
        if (hipEventRecord(plan->done[slot], stream) != hipSuccess) return OSERVE_ERR_DEVICE;
    } else if (oserve::launch_prefill(pp, plan->list.geo.head_dim, n_items, stream, nullptr, plan->done[slot]) != hipSuccess) {
        return OSERVE_ERR_DEVICE;
    }
    plan->slot_used[slot] = true;
    return OSERVE_OK;
}

oserve_status_t oserve_prefill_plan_enable_timing(oserve_prefill_plan_t* plan, int32_t enable) {
    if (!plan) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.set_enabled(enable != 0) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

oserve_status_t oserve_prefill_plan_kernel_ms(oserve_prefill_plan_t* plan, float* mean_ms, int32_t* count) {
    if (!plan || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.mean(mean_ms, count) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

}  // extern "C"
