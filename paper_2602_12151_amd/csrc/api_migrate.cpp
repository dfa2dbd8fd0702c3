// C ABI of the KV-block migration copies (declared in include/oserve.h).  Host code only; the
// kernel lives in migrate.hip.
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <new>
#include <vector>

#include "host_util.h"
#include "kernels.h"
#include "oserve.h"

struct oserve_kv_migration {
    int32_t device_id = -1;
    int32_t num_requests = 0;
    int32_t page_size = 0;
    int32_t max_request_pages = 0;
    int64_t num_pages = 0;
    std::vector<int32_t> offsets;   // [R + 1]
    int32_t* dev = nullptr;         // [num_pages][4]: source table row, request, page within the request, 0
    oserve::KernelTimer<1> timer;   // optional copy-kernel timing (the latest launch)
};

namespace {

using Guard = oserve::DeviceGuard;

void release(oserve_kv_migration* m) {
    m->timer.destroy();
    if (m->dev) (void)hipFree(m->dev);
}

oserve_status_t run(oserve_kv_migration* m, bool gather, const void* k_src, const void* v_src, void* k_dst,
                    void* v_dst, const int32_t* table, int32_t table_stride, bool use_rows, int32_t pool_heads,
                    int32_t head_begin, int32_t num_heads, int32_t head_dim, void* stream_v) {
    if (!m || !k_src || !v_src || !k_dst || !v_dst || !table) return OSERVE_ERR_NULL;
    if (m->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    if (pool_heads < 1 || head_begin < 0 || num_heads < 1 || head_begin + num_heads > pool_heads) return OSERVE_ERR_SHAPE;
    if (head_dim < 8 || head_dim % 8 != 0 || table_stride < m->max_request_pages) return OSERVE_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(k_src) | reinterpret_cast<uintptr_t>(v_src) |
         reinterpret_cast<uintptr_t>(k_dst) | reinterpret_cast<uintptr_t>(v_dst)) & 15u)
        return OSERVE_ERR_ALIGNMENT;
    Guard guard(m->device_id);
    if (!guard.ok) return OSERVE_ERR_DEVICE;
    if (m->timer.enabled && !m->timer.collect(0)) return OSERVE_ERR_DEVICE;
    oserve::MigrateParams p{};
    p.k_src = k_src; p.v_src = v_src; p.k_dst = k_dst; p.v_dst = v_dst;
    p.block_table = table;
    p.table_stride = table_stride;
    p.page_refs = m->dev;
    p.use_source_rows = use_rows ? 1 : 0;
    p.num_pages = m->num_pages;
    p.pool_heads = pool_heads;
    p.head_begin = head_begin;
    p.num_heads = num_heads;
    p.unit_chunks = m->page_size * head_dim * 2 / 16;
    if (oserve::launch_kv_migrate(p, gather, static_cast<hipStream_t>(stream_v),
                                  m->timer.begin_of(0), m->timer.end_of(0)) != hipSuccess)
        return OSERVE_ERR_DEVICE;
    m->timer.mark(0);
    return OSERVE_OK;
}

}  // namespace

extern "C" {

oserve_status_t oserve_kv_migration_create(const int32_t* context_lens_host, const int32_t* table_rows_host,
                                           int32_t num_requests, int32_t page_size, int32_t device_id,
                                           oserve_kv_migration_t** out) {
    if (!out) return OSERVE_ERR_NULL;
    *out = nullptr;
    if (!context_lens_host || !table_rows_host) return OSERVE_ERR_NULL;
    if (num_requests < 1 || num_requests > (1 << 20) || device_id < -1) return OSERVE_ERR_SHAPE;
    if (page_size != 16 && page_size != 32 && page_size != 64) return OSERVE_ERR_SHAPE;
    oserve_kv_migration* m = new (std::nothrow) oserve_kv_migration();
    if (!m) return OSERVE_ERR_DEVICE;
    m->device_id = device_id;
    m->num_requests = num_requests;
    m->page_size = page_size;
    m->offsets.resize(static_cast<size_t>(num_requests) + 1);
    int64_t total = 0;
    for (int32_t r = 0; r < num_requests; ++r) {
        if (context_lens_host[r] < 1 || table_rows_host[r] < 0) { delete m; return OSERVE_ERR_CONTEXT_LEN; }
        m->offsets[r] = static_cast<int32_t>(total);
        const int32_t pages = (context_lens_host[r] + page_size - 1) / page_size;
        if (pages > m->max_request_pages) m->max_request_pages = pages;
        total += pages;
        if (total > (1ll << 30)) { delete m; return OSERVE_ERR_SHAPE; }
    }
    m->offsets[num_requests] = static_cast<int32_t>(total);
    m->num_pages = total;
    if (device_id >= 0) {
        int n_dev = 0;
        bool ok = hipGetDeviceCount(&n_dev) == hipSuccess && device_id < n_dev;
        if (ok) {
            Guard guard(device_id);
            ok = guard.ok;
            // per staging page, which table entry names it: the copy kernel starts from one load
            std::vector<int32_t> refs(4 * static_cast<size_t>(total));
            for (int32_t r = 0; r < num_requests; ++r)
                for (int32_t s = m->offsets[r]; s < m->offsets[r + 1]; ++s) {
                    int32_t* e = &refs[4 * static_cast<size_t>(s)];
                    e[0] = table_rows_host[r]; e[1] = r; e[2] = s - m->offsets[r]; e[3] = 0;
                }
            const size_t bytes = refs.size() * sizeof(int32_t);
            ok = ok && hipMalloc(reinterpret_cast<void**>(&m->dev), bytes) == hipSuccess;
            ok = ok && hipMemcpy(m->dev, refs.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
            ok = ok && m->timer.create();
        }
        if (!ok) { release(m); delete m; return OSERVE_ERR_DEVICE; }
    }
    *out = m;
    return OSERVE_OK;
}

void oserve_kv_migration_destroy(oserve_kv_migration_t* m) {
    if (!m) return;
    if (m->device_id >= 0) release(m);
    delete m;
}

int64_t oserve_kv_migration_num_pages(const oserve_kv_migration_t* m) { return m->num_pages; }

oserve_status_t oserve_kv_migration_request(const oserve_kv_migration_t* m, int32_t r, int32_t* first_page,
                                            int32_t* num_pages) {
    if (!m) return OSERVE_ERR_NULL;
    if (r < 0 || r >= m->num_requests) return OSERVE_ERR_SHAPE;
    if (first_page) *first_page = m->offsets[r];
    if (num_pages) *num_pages = m->offsets[r + 1] - m->offsets[r];
    return OSERVE_OK;
}

oserve_status_t oserve_kv_gather(oserve_kv_migration_t* m, const void* k_pool, const void* v_pool,
                                 const int32_t* block_table, int32_t max_pages_per_seq, int32_t pool_kv_heads,
                                 int32_t head_begin, int32_t num_heads, int32_t head_dim, void* k_stage,
                                 void* v_stage, void* stream) {
    return run(m, true, k_pool, v_pool, k_stage, v_stage, block_table, max_pages_per_seq, true, pool_kv_heads,
               head_begin, num_heads, head_dim, stream);
}

oserve_status_t oserve_kv_scatter(oserve_kv_migration_t* m, const void* k_stage, const void* v_stage,
                                  const int32_t* target_block_table, int32_t max_pages_per_seq,
                                  int32_t pool_kv_heads, int32_t head_begin, int32_t num_heads, int32_t head_dim,
                                  void* k_pool, void* v_pool, void* stream) {
    return run(m, false, k_stage, v_stage, k_pool, v_pool, target_block_table, max_pages_per_seq, false,
               pool_kv_heads, head_begin, num_heads, head_dim, stream);
}

oserve_status_t oserve_kv_migration_enable_timing(oserve_kv_migration_t* m, int32_t enable) {
    if (!m) return OSERVE_ERR_NULL;
    if (m->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return m->timer.set_enabled(enable != 0) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

oserve_status_t oserve_kv_migration_kernel_ms(oserve_kv_migration_t* m, float* mean_ms, int32_t* count) {
    if (!m || !mean_ms || !count) return OSERVE_ERR_NULL;
    if (m->device_id < 0) return OSERVE_ERR_PLAN_MISMATCH;
    return m->timer.mean(mean_ms, count) ? OSERVE_OK : OSERVE_ERR_DEVICE;
}

}  // extern "C"
