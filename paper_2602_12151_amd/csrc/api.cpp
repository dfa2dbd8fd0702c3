// C ABI of the library (declared in include/oserve.h): plan objects and the
// launch call.  Host code only; the kernels live in kernels.hip.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "kernels.h"
#include "oserve.h"
#include "plan.h"

using oserve::RunRecord;
using oserve::SplitPlan;

struct oserve_plan {
    SplitPlan host;
    int32_t device_id = -1;
    // pinned staging for the upload of run records + request info: OSERVE_PLAN_RING slots
    char* staging = nullptr;
    char* staging_dev = nullptr;   // the same memory as the device addresses it
    size_t staging_slot_bytes = 0;
    hipEvent_t upload_done[OSERVE_PLAN_RING] = {};
    bool slot_used[OSERVE_PLAN_RING] = {};
    int next_slot = 0;
    // optional split-kernel timing
    bool timing = false;
    hipEvent_t t_begin[OSERVE_PLAN_RING] = {}, t_end[OSERVE_PLAN_RING] = {};
    bool t_pending[OSERVE_PLAN_RING] = {};
    double t_sum_ms = 0.0;
    int64_t t_count = 0;
};

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        target = dev;
    }
    ~DeviceGuard() {
        if (ok && prev != target) (void)hipSetDevice(prev);
    }
    int target = -1;
};

void release_device_state(oserve_plan* pl) {
    for (int i = 0; i < OSERVE_PLAN_RING; ++i) {
        if (pl->upload_done[i]) (void)hipEventDestroy(pl->upload_done[i]);
        if (pl->t_begin[i]) (void)hipEventDestroy(pl->t_begin[i]);
        if (pl->t_end[i]) (void)hipEventDestroy(pl->t_end[i]);
    }
    if (pl->staging) (void)hipHostFree(pl->staging);
}

// Fold a finished timing slot into the running mean.  Blocks until the slot's end event.
bool collect_timing(oserve_plan* pl, int slot) {
    if (!pl->t_pending[slot]) return true;
    if (hipEventSynchronize(pl->t_end[slot]) != hipSuccess) return false;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, pl->t_begin[slot], pl->t_end[slot]) != hipSuccess) return false;
    pl->t_sum_ms += ms;
    pl->t_count += 1;
    pl->t_pending[slot] = false;
    return true;
}

}  // namespace

extern "C" {

oserve_status_t oserve_plan_create(const int32_t* context_lens_host, int32_t batch,
                                   int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                                   int32_t page_size, int32_t max_pages_per_seq,
                                   int32_t split_tokens, int32_t device_id, int32_t capacity,
                                   oserve_plan_t** plan_out) {
    if (!plan_out) return OSERVE_ERR_NULL;
    *plan_out = nullptr;
    if (!context_lens_host) return OSERVE_ERR_NULL;
    const oserve::Geometry geo{num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq};
    oserve_status_t st = SplitPlan::check_geometry(geo, batch, capacity, split_tokens);
    if (st != OSERVE_OK) return st;
    if (device_id < -1) return OSERVE_ERR_SHAPE;

    oserve_plan* pl = new (std::nothrow) oserve_plan();
    if (!pl) return OSERVE_ERR_DEVICE;
    pl->host.geo = geo;
    pl->host.capacity = capacity;
    pl->host.split_pages_user = split_tokens / oserve::kTileTokens;
    pl->host.reserve();
    pl->staging_slot_bytes = (static_cast<size_t>(pl->host.max_runs()) * sizeof(RunRecord) +
                              static_cast<size_t>(capacity) * sizeof(oserve::RequestInfo) + 16 + 255) & ~static_cast<size_t>(255);
    if (const char* e = getenv("OSERVE_PLAN_TUNING")) {  // experiments: "items_per_slot_x4,tail_slots_x16,max_split_pages"
        int a = 0, b = 0, c = 0;
        if (sscanf(e, "%d,%d,%d", &a, &b, &c) == 3 && a > 0 && b >= 0 && c >= 12)
            pl->host.tuning = oserve::PlanTuning{a, b, c};
    }
    pl->device_id = device_id;

    if (device_id >= 0) {
        int n_dev = 0, cus = 0;
        bool ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev;
        ok = ok && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device_id) == hipSuccess;
        if (ok) {
            DeviceGuard guard(device_id);
            ok = guard.ok;
            ok = ok && hipHostMalloc(reinterpret_cast<void**>(&pl->staging),
                                     pl->staging_slot_bytes * OSERVE_PLAN_RING,
                                     hipHostMallocDefault) == hipSuccess;
            ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&pl->staging_dev), pl->staging, 0) == hipSuccess;
            for (int i = 0; ok && i < OSERVE_PLAN_RING; ++i) {
                ok = hipEventCreateWithFlags(&pl->upload_done[i], hipEventDisableTiming) == hipSuccess;
                ok = ok && hipEventCreate(&pl->t_begin[i]) == hipSuccess;
                ok = ok && hipEventCreate(&pl->t_end[i]) == hipSuccess;
            }
        }
        if (!ok) {
            release_device_state(pl);
            delete pl;
            return OSERVE_ERR_DEVICE;
        }
        if (cus > 0) pl->host.num_cus = cus;
    }

    st = pl->host.build(context_lens_host, batch);
    if (st != OSERVE_OK) {
        if (device_id >= 0) release_device_state(pl);
        delete pl;
        return st;
    }
    *plan_out = pl;
    return OSERVE_OK;
}

oserve_status_t oserve_plan_update(oserve_plan_t* plan, const int32_t* context_lens_host, int32_t batch) {
    if (!plan || !context_lens_host) return OSERVE_ERR_NULL;
    return plan->host.build(context_lens_host, batch);
}

void oserve_plan_destroy(oserve_plan_t* plan) {
    if (!plan) return;
    if (plan->device_id >= 0) release_device_state(plan);
    delete plan;
}

int32_t oserve_plan_batch(const oserve_plan_t* plan) { return plan->host.batch; }
int32_t oserve_plan_num_work_items(const oserve_plan_t* plan) { return plan->host.num_items; }
int32_t oserve_plan_split_pages(const oserve_plan_t* plan) { return plan->host.split_pages; }

oserve_status_t oserve_plan_request(const oserve_plan_t* plan, int32_t b, int32_t* num_splits,
                                    int32_t* max_split_pages) {
    if (!plan) return OSERVE_ERR_NULL;
    if (b < 0 || b >= plan->host.batch) return OSERVE_ERR_SHAPE;
    if (num_splits) *num_splits = plan->host.req_info[b].num_splits;
    if (max_split_pages) *max_split_pages = plan->host.split_pages;
    return OSERVE_OK;
}

int32_t oserve_plan_num_runs(const oserve_plan_t* plan) { return static_cast<int32_t>(plan->host.records.size()); }

oserve_status_t oserve_plan_run(const oserve_plan_t* plan, int32_t i, int32_t fields[8]) {
    if (!plan || !fields) return OSERVE_ERR_NULL;
    if (i < 0 || i >= static_cast<int32_t>(plan->host.records.size())) return OSERVE_ERR_SHAPE;
    std::memcpy(fields, &plan->host.records[i], sizeof(RunRecord));
    return OSERVE_OK;
}

size_t oserve_plan_workspace_bytes(const oserve_plan_t* plan) {
    const SplitPlan& hp = plan->host;
    return hp.layout(hp.num_items, hp.num_row_groups, static_cast<int64_t>(hp.records.size()), hp.batch).total;
}

size_t oserve_plan_workspace_bytes_max(const oserve_plan_t* plan) {
    const SplitPlan& hp = plan->host;
    const int64_t items = hp.max_items();
    return hp.layout(items, items / hp.geo.num_kv_heads, hp.max_runs(), hp.capacity).total;
}

oserve_status_t oserve_paged_decode_attn(oserve_plan_t* plan, void* workspace, size_t workspace_bytes,
                                         const void* q, const void* k_pages, const void* v_pages,
                                         const int32_t* block_table, const int32_t* context_lens,
                                         float scale, float* out, void* stream_v) {
    if (!plan || !workspace || !q || !k_pages || !v_pages || !block_table || !context_lens || !out)
        return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    const SplitPlan& hp = plan->host;
    const int64_t num_runs = static_cast<int64_t>(hp.records.size());
    const oserve::WorkspaceLayout lay = hp.layout(hp.num_items, hp.num_row_groups, num_runs, hp.batch);
    if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return OSERVE_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pages) |
         reinterpret_cast<uintptr_t>(v_pages) | reinterpret_cast<uintptr_t>(out)) & 15u)
        return OSERVE_ERR_SHAPE;

    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    DeviceGuard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;

    // stage the records in the next pinned slot (waits only if that slot's last upload is still pending)
    const int slot = plan->next_slot;
    plan->next_slot = (slot + 1) % OSERVE_PLAN_RING;
    if (plan->slot_used[slot] && hipEventSynchronize(plan->upload_done[slot]) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    if (plan->timing && !collect_timing(plan, slot)) return OSERVE_ERR_DEVICE;
    // slot layout: [run records][request info]; both 16-byte aligned
    const size_t slot_off = static_cast<size_t>(slot) * plan->staging_slot_bytes;
    const size_t info_off = sizeof(RunRecord) * static_cast<size_t>(num_runs);
    std::memcpy(plan->staging + slot_off, hp.records.data(), info_off);
    std::memcpy(plan->staging + slot_off + info_off, hp.req_info.data(), sizeof(oserve::RequestInfo) * hp.batch);
    char* ws = static_cast<char*>(workspace);
    oserve::ExpandParams ep{};
    ep.records_host = reinterpret_cast<const RunRecord*>(plan->staging_dev + slot_off);
    ep.num_runs = static_cast<int32_t>(num_runs);
    ep.req_info_host = reinterpret_cast<const oserve::RequestInfo*>(plan->staging_dev + slot_off + info_off);
    ep.req_info = reinterpret_cast<oserve::RequestInfo*>(ws + lay.req_info_off);
    ep.batch = hp.batch;
    ep.items = reinterpret_cast<oserve::ItemDesc*>(ws + lay.items_off);
    ep.num_kv_heads = hp.geo.num_kv_heads;
    ep.kv_heads_magic = static_cast<uint32_t>((1ull << 32) / static_cast<uint32_t>(hp.geo.num_kv_heads)) + 1u;
    if (oserve::launch_expand(ep, stream, plan->upload_done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    plan->slot_used[slot] = true;

    oserve::SplitParams sp{};
    sp.items = ep.items;
    sp.q = static_cast<const uint16_t*>(q);
    sp.k_pages = static_cast<const uint16_t*>(k_pages);
    sp.v_pages = static_cast<const uint16_t*>(v_pages);
    sp.block_table = block_table;
    sp.context_lens = context_lens;
    sp.out = out;
    sp.partial_o = reinterpret_cast<float*>(ws + lay.partial_o_off);
    sp.partial_ml = reinterpret_cast<float*>(ws + lay.partial_ml_off);
    sp.scale_log2e = scale * 1.44269504088896340736f;
    sp.num_q_heads = hp.geo.num_q_heads;
    sp.num_kv_heads = hp.geo.num_kv_heads;
    sp.group = hp.geo.group();
    sp.max_pages_per_seq = hp.geo.max_pages_per_seq;
    sp.tile_shift = hp.geo.page_size == 64 ? 2 : hp.geo.page_size == 32 ? 1 : 0;

    if (oserve::launch_split(sp, hp.geo.head_dim, hp.num_items, stream,
                             plan->timing ? plan->t_begin[slot] : nullptr,
                             plan->timing ? plan->t_end[slot] : nullptr) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    if (plan->timing) plan->t_pending[slot] = true;

    oserve::MergeParams mp{};
    mp.req_info = reinterpret_cast<const oserve::RequestInfo*>(ws + lay.req_info_off);
    mp.partial_o = sp.partial_o;
    mp.partial_ml = sp.partial_ml;
    mp.out = out;
    mp.num_q_heads = sp.num_q_heads;
    if (hp.num_row_groups > hp.batch) {  // at least one request is split
        if (oserve::launch_merge(mp, hp.geo.head_dim, hp.batch, stream) != hipSuccess)
            return OSERVE_ERR_DEVICE;
    }
    return OSERVE_OK;
}

oserve_status_t oserve_plan_enable_timing(oserve_plan_t* plan, int32_t enable) {
    if (!plan) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    for (int i = 0; i < OSERVE_PLAN_RING; ++i)
        if (!collect_timing(plan, i)) return OSERVE_ERR_DEVICE;
    plan->timing = enable != 0;
    plan->t_sum_ms = 0.0;
    plan->t_count = 0;
    return OSERVE_OK;
}

oserve_status_t oserve_plan_split_kernel_ms(oserve_plan_t* plan, float* mean_ms, int32_t* count) {
    if (!plan || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    for (int i = 0; i < OSERVE_PLAN_RING; ++i)
        if (!collect_timing(plan, i)) return OSERVE_ERR_DEVICE;
    *count = static_cast<int32_t>(plan->t_count);
    *mean_ms = plan->t_count ? static_cast<float>(plan->t_sum_ms / plan->t_count) : 0.f;
    return OSERVE_OK;
}

const char* oserve_status_string(oserve_status_t status) {
    switch (status) {
        case OSERVE_OK: return "ok";
        case OSERVE_ERR_NULL: return "null pointer";
        case OSERVE_ERR_SHAPE: return "unsupported shape or alignment";
        case OSERVE_ERR_CONTEXT_LEN: return "context length out of range";
        case OSERVE_ERR_WORKSPACE: return "workspace too small or misaligned";
        case OSERVE_ERR_PLAN_MISMATCH: return "plan does not match the call";
        case OSERVE_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
