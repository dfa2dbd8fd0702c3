// C ABI of the library (declared in include/oserve.h): plan objects and the
// launch call.  Host code only; the kernels live in kernels.hip.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <algorithm>
#include <cstring>
#include <new>

#include "decode_launch.h"
#include "host_util.h"
#include "kernels.h"
#include "oserve.h"
#include "plan.h"

using oserve::DeviceGuard;
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
    oserve::KernelTimer<OSERVE_PLAN_RING> timer;   // optional split-kernel timing
    int next_timer_slot = 0;
    // oserve_plan_stage: which build of the plan was expanded into which workspace
    uint64_t generation = 0;            // grows with every successful build
    uint64_t staged_generation = 0;     // 0 = nothing staged
    const void* staged_workspace = nullptr;
};

namespace {

void release_device_state(oserve_plan* pl) {
    for (int i = 0; i < OSERVE_PLAN_RING; ++i) {
        if (pl->upload_done[i]) (void)hipEventDestroy(pl->upload_done[i]);
    }
    pl->timer.destroy();
    if (pl->staging) (void)hipHostFree(pl->staging);
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
    pl->device_id = device_id;

    if (device_id >= 0) {
        int n_dev = 0;
        oserve::DeviceFacts facts;
        bool ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev;
        ok = ok && oserve::query_device_facts(device_id, &facts);
        if (ok) {
            DeviceGuard guard(device_id);
            ok = guard.ok;
            ok = ok && hipHostMalloc(reinterpret_cast<void**>(&pl->staging),
                                     pl->staging_slot_bytes * OSERVE_PLAN_RING,
                                     hipHostMallocDefault) == hipSuccess;
            ok = ok && hipHostGetDevicePointer(reinterpret_cast<void**>(&pl->staging_dev), pl->staging, 0) == hipSuccess;
            for (int i = 0; ok && i < OSERVE_PLAN_RING; ++i) {
                ok = hipEventCreateWithFlags(&pl->upload_done[i], hipEventDisableTiming) == hipSuccess;
            }
            ok = ok && pl->timer.create();
        }
        if (!ok) {
            release_device_state(pl);
            delete pl;
            return OSERVE_ERR_DEVICE;
        }
        pl->host.wave_slots = facts.compute_units * facts.simds_per_cu;
    }

    st = pl->host.build(context_lens_host, batch);
    if (st != OSERVE_OK) {
        if (device_id >= 0) release_device_state(pl);
        delete pl;
        return st;
    }
    pl->generation = 1;
    *plan_out = pl;
    return OSERVE_OK;
}

oserve_status_t oserve_plan_update(oserve_plan_t* plan, const int32_t* context_lens_host, int32_t batch) {
    if (!plan || !context_lens_host) return OSERVE_ERR_NULL;
    const oserve_status_t st = plan->host.build(context_lens_host, batch);
    if (st == OSERVE_OK) plan->generation += 1;   // descriptors staged for the previous build are stale now
    return st;
}

void oserve_plan_destroy(oserve_plan_t* plan) {
    if (!plan) return;
    if (plan->device_id >= 0) release_device_state(plan);
    delete plan;
}

int32_t oserve_plan_batch(const oserve_plan_t* plan) { return plan->host.batch; }
int32_t oserve_plan_num_work_items(const oserve_plan_t* plan) { return plan->host.num_items; }
int32_t oserve_plan_split_pages(const oserve_plan_t* plan) { return plan->host.split_pages; }
int32_t oserve_plan_split_tokens(const oserve_plan_t* plan) { return plan->host.split_pages * oserve::kTileTokens; }

oserve_status_t oserve_plan_request(const oserve_plan_t* plan, int32_t b, int32_t* num_splits,
                                    int32_t* max_split_pages) {
    if (!plan) return OSERVE_ERR_NULL;
    if (b < 0 || b >= plan->host.batch) return OSERVE_ERR_SHAPE;
    if (num_splits) *num_splits = plan->host.req_info[b].num_splits;
    if (max_split_pages) {
        int32_t largest = 0;
        for (const RunRecord& r : plan->host.records)
            if (r.request == b) largest = std::max(largest, std::min(r.pages_per_split, r.page_end - r.page_begin));
        *max_split_pages = largest;
    }
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
    return hp.layout(hp.num_items, hp.num_row_groups, hp.batch).total;
}

size_t oserve_plan_workspace_bytes_max(const oserve_plan_t* plan) {
    const SplitPlan& hp = plan->host;
    const int64_t items = hp.max_items();
    return hp.layout(items, items / hp.geo.num_kv_heads, hp.capacity).total;
}

}  // extern "C"

namespace oserve {

namespace {

oserve_status_t check_workspace(const oserve_plan_t* plan, const void* workspace, size_t workspace_bytes,
                                WorkspaceLayout* lay) {
    const SplitPlan& hp = plan->host;
    *lay = hp.layout(hp.num_items, hp.num_row_groups, hp.batch);
    if (workspace_bytes < lay->total || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return OSERVE_ERR_WORKSPACE;
    return OSERVE_OK;
}

// Records staged in the plan's next pinned slot, then the expand kernel that turns them into the
// work-item descriptors and request records of `workspace`.
oserve_status_t enqueue_expand(oserve_plan_t* plan, const WorkspaceLayout& lay, void* workspace, hipStream_t stream) {
    const SplitPlan& hp = plan->host;
    const int64_t num_runs = static_cast<int64_t>(hp.records.size());
    // waits only if that slot's last upload is still pending
    const int slot = plan->next_slot;
    plan->next_slot = (slot + 1) % OSERVE_PLAN_RING;
    if (plan->slot_used[slot] && hipEventSynchronize(plan->upload_done[slot]) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    // slot layout: [run records][request info]; both 16-byte aligned
    const size_t slot_off = static_cast<size_t>(slot) * plan->staging_slot_bytes;
    const size_t info_off = sizeof(RunRecord) * static_cast<size_t>(num_runs);
    std::memcpy(plan->staging + slot_off, hp.records.data(), info_off);
    std::memcpy(plan->staging + slot_off + info_off, hp.req_info.data(), sizeof(RequestInfo) * hp.batch);
    char* ws = static_cast<char*>(workspace);
    ExpandParams ep{};
    ep.records_host = reinterpret_cast<const RunRecord*>(plan->staging_dev + slot_off);
    ep.num_runs = static_cast<int32_t>(num_runs);
    ep.req_info_host = reinterpret_cast<const RequestInfo*>(plan->staging_dev + slot_off + info_off);
    ep.req_info = reinterpret_cast<RequestInfo*>(ws + lay.req_info_off);
    ep.batch = hp.batch;
    ep.items = reinterpret_cast<ItemDesc*>(ws + lay.items_off);
    ep.num_kv_heads = hp.geo.num_kv_heads;
    ep.kv_heads_magic = static_cast<uint32_t>((1ull << 32) / static_cast<uint32_t>(hp.geo.num_kv_heads)) + 1u;
    if (launch_expand(ep, stream, plan->upload_done[slot]) != hipSuccess) return OSERVE_ERR_DEVICE;
    plan->slot_used[slot] = true;
    return OSERVE_OK;
}

// The split kernel and (if any request is split) the merge kernel over descriptors that are in `workspace`.
oserve_status_t enqueue_split_and_merge(oserve_plan_t* plan, const WorkspaceLayout& lay, void* workspace,
                                        const void* q, const void* k_pages, const void* v_pages,
                                        const int32_t* block_table, const int32_t* context_lens, float scale,
                                        float* out, hipStream_t stream) {
    const SplitPlan& hp = plan->host;
    char* ws = static_cast<char*>(workspace);
    const int tslot = plan->next_timer_slot;
    plan->next_timer_slot = (tslot + 1) % OSERVE_PLAN_RING;
    if (plan->timer.enabled && !plan->timer.collect(tslot)) return OSERVE_ERR_DEVICE;

    SplitParams sp{};
    sp.items = reinterpret_cast<const ItemDesc*>(ws + lay.items_off);
    sp.req_info = reinterpret_cast<const RequestInfo*>(ws + lay.req_info_off);
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

    if (launch_split(sp, hp.geo.head_dim, hp.num_items, stream, plan->timer.begin_of(tslot),
                     plan->timer.end_of(tslot)) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    plan->timer.mark(tslot);

    MergeParams mp{};
    mp.req_info = sp.req_info;
    mp.partial_o = sp.partial_o;
    mp.partial_ml = sp.partial_ml;
    mp.out = out;
    mp.num_q_heads = sp.num_q_heads;
    if (hp.needs_merge) {  // at least one request is split
        if (launch_merge(mp, hp.geo.head_dim, hp.batch, stream) != hipSuccess) return OSERVE_ERR_DEVICE;
    }
    return OSERVE_OK;
}

bool misaligned(const void* q, const void* k_pages, const void* v_pages, const void* out) {
    return ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pages) |
             reinterpret_cast<uintptr_t>(v_pages) | reinterpret_cast<uintptr_t>(out)) & 15u) != 0;
}

}  // namespace

// The whole decode step on `stream`: the expand, split and (if any request is split) merge kernels.
// Allocates nothing.
oserve_status_t decode_launch(oserve_plan_t* plan, void* workspace, size_t workspace_bytes, const void* q,
                              const void* k_pages, const void* v_pages, const int32_t* block_table,
                              const int32_t* context_lens, float scale, float* out, void* stream_v) {
    if (!plan || !workspace || !q || !k_pages || !v_pages || !block_table || !context_lens || !out)
        return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    WorkspaceLayout lay;
    oserve_status_t st = check_workspace(plan, workspace, workspace_bytes, &lay);
    if (st != OSERVE_OK) return st;
    if (misaligned(q, k_pages, v_pages, out)) return OSERVE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    DeviceGuard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;
    if (workspace == plan->staged_workspace) plan->staged_generation = 0;   // re-expanded below: the same content, but staged no longer
    st = enqueue_expand(plan, lay, workspace, stream);
    if (st != OSERVE_OK) return st;
    return enqueue_split_and_merge(plan, lay, workspace, q, k_pages, v_pages, block_table, context_lens, scale, out, stream);
}

size_t decode_workspace_bytes(const oserve_plan_t* plan) { return oserve_plan_workspace_bytes(plan); }
int decode_plan_device(const oserve_plan_t* plan) { return plan->device_id; }

}  // namespace oserve

extern "C" {

oserve_status_t oserve_paged_decode_attn(oserve_plan_t* plan, void* workspace, size_t workspace_bytes,
                                         const void* q, const void* k_pages, const void* v_pages,
                                         const int32_t* block_table, const int32_t* context_lens,
                                         float scale, float* out, void* stream) {
    return oserve::decode_launch(plan, workspace, workspace_bytes, q, k_pages, v_pages, block_table,
                                 context_lens, scale, out, stream);
}

oserve_status_t oserve_plan_stage(oserve_plan_t* plan, void* workspace, size_t workspace_bytes, void* stream_v) {
    if (!plan || !workspace) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    oserve::WorkspaceLayout lay;
    const oserve_status_t st = oserve::check_workspace(plan, workspace, workspace_bytes, &lay);
    if (st != OSERVE_OK) return st;
    oserve::DeviceGuard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;
    plan->staged_generation = 0;
    const oserve_status_t se = oserve::enqueue_expand(plan, lay, workspace, static_cast<hipStream_t>(stream_v));
    if (se != OSERVE_OK) return se;
    plan->staged_generation = plan->generation;
    plan->staged_workspace = workspace;
    return OSERVE_OK;
}

oserve_status_t oserve_paged_decode_attn_staged(oserve_plan_t* plan, void* workspace, size_t workspace_bytes,
                                                const void* q, const void* k_pages, const void* v_pages,
                                                const int32_t* block_table, const int32_t* context_lens,
                                                float scale, float* out, void* stream_v) {
    if (!plan || !workspace || !q || !k_pages || !v_pages || !block_table || !context_lens || !out)
        return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    // the descriptors in `workspace` must be those of the plan as it is now
    if (plan->staged_generation == 0 || plan->staged_generation != plan->generation || plan->staged_workspace != workspace)
        return OSERVE_ERR_PLAN_MISMATCH;
    oserve::WorkspaceLayout lay;
    const oserve_status_t st = oserve::check_workspace(plan, workspace, workspace_bytes, &lay);
    if (st != OSERVE_OK) return st;
    if (oserve::misaligned(q, k_pages, v_pages, out)) return OSERVE_ERR_ALIGNMENT;
    oserve::DeviceGuard guard(plan->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;
    return oserve::enqueue_split_and_merge(plan, lay, workspace, q, k_pages, v_pages, block_table, context_lens,
                                           scale, out, static_cast<hipStream_t>(stream_v));
}

oserve_status_t oserve_plan_enable_timing(oserve_plan_t* plan, int32_t enable) {
    if (!plan) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.set_enabled(enable != 0) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

oserve_status_t oserve_plan_split_kernel_ms(oserve_plan_t* plan, float* mean_ms, int32_t* count) {
    if (!plan || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (plan->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return plan->timer.mean(mean_ms, count) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

const char* oserve_status_string(oserve_status_t status) {
    switch (status) {
        case OSERVE_OK: return "ok";
        case OSERVE_ERR_NULL: return "null pointer";
        case OSERVE_ERR_SHAPE: return "unsupported shape";
        case OSERVE_ERR_CONTEXT_LEN: return "context length out of range";
        case OSERVE_ERR_WORKSPACE: return "workspace too small or misaligned";
        case OSERVE_ERR_PLAN_MISMATCH: return "plan does not match the call";
        case OSERVE_ERR_DEVICE: return "HIP runtime error";
        case OSERVE_ERR_ALIGNMENT: return "misaligned device pointer";
    }
    return "unknown status";
}

}  // extern "C"
