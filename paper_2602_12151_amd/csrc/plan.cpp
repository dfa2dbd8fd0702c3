// Host-side planning: sizes the per-request sequence splits of a mixed-length
// batch so that short and long requests fill the device together (the
// spatially heterogeneous batch of paper section 1 (i) / section 2).
#include "plan.h"

#include <algorithm>
#include <numeric>

namespace oserve {

oserve_status_t SplitPlan::check_geometry(const Geometry& g, int32_t batch, int32_t capacity,
                                          int32_t split_tokens) {
    if (g.num_q_heads < 1 || g.num_kv_heads < 1 || g.num_q_heads % g.num_kv_heads != 0)
        return OSERVE_ERR_SHAPE;
    if (g.group() > 16) return OSERVE_ERR_SHAPE;
    if (g.head_dim != 64 && g.head_dim != 128) return OSERVE_ERR_SHAPE;
    if (g.page_size != 16) return OSERVE_ERR_SHAPE;
    if (g.max_pages_per_seq < 1 || batch < 1 || capacity < batch) return OSERVE_ERR_SHAPE;
    if (split_tokens < 0 || split_tokens % g.page_size != 0) return OSERVE_ERR_SHAPE;
    return OSERVE_OK;
}

int64_t SplitPlan::max_items() const {
    const int64_t per_req_max =
        split_pages_user > 0
            ? (static_cast<int64_t>(geo.max_pages_per_seq) + split_pages_user - 1) / split_pages_user
            : 0;
    if (split_pages_user > 0) return per_req_max * capacity * geo.num_kv_heads;
    // automatic: C >= total_units / target  =>  sum_b ceil(N_b / C) * Hkv <= target + capacity * Hkv
    return static_cast<int64_t>(num_cus) * kWavesPerCu * kOversubscribe +
           static_cast<int64_t>(capacity) * geo.num_kv_heads;
}

WorkspaceLayout SplitPlan::layout(int64_t items, int32_t n) const {
    auto align = [](size_t x) { return (x + 255) & ~static_cast<size_t>(255); };
    WorkspaceLayout w{};
    w.records_off = 0;
    w.partial_o_off = align(static_cast<size_t>(n) * sizeof(RequestRecord));
    const size_t rows = static_cast<size_t>(items) * geo.group();
    w.partial_ml_off = w.partial_o_off + align(rows * geo.head_dim * sizeof(float));
    w.total = w.partial_ml_off + align(rows * 2 * sizeof(float));
    return w;
}

oserve_status_t SplitPlan::build(const int32_t* lens, int32_t n) {
    if (!lens) return OSERVE_ERR_NULL;
    if (n < 1 || n > capacity) return OSERVE_ERR_PLAN_MISMATCH;
    const int64_t max_len = static_cast<int64_t>(geo.max_pages_per_seq) * geo.page_size;
    int64_t total_pages = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (lens[b] < 1 || lens[b] > max_len) return OSERVE_ERR_CONTEXT_LEN;
        total_pages += (lens[b] + geo.page_size - 1) / geo.page_size;
    }

    int32_t c = split_pages_user;
    if (c == 0) {
        const int64_t units = total_pages * geo.num_kv_heads;
        const int64_t target = static_cast<int64_t>(num_cus) * kWavesPerCu * kOversubscribe;
        c = static_cast<int32_t>(std::max<int64_t>(kMinSplitPages, (units + target - 1) / target));
    }

    std::vector<RequestRecord>& recs = scratch_records;   // reserved to capacity: no allocation here
    std::vector<int32_t>& pos = scratch_position;
    recs.resize(static_cast<size_t>(n));
    pos.resize(static_cast<size_t>(n));
    for (int32_t b = 0; b < n; ++b) {
        const int32_t pages = (lens[b] + geo.page_size - 1) / geo.page_size;
        const int32_t splits = (pages + c - 1) / c;
        recs[b] = RequestRecord{b, 0, splits, (pages + splits - 1) / splits, pages, {0, 0, 0}};
    }
    // longest split first; ties by request index so the order is deterministic
    std::stable_sort(recs.begin(), recs.end(), [](const RequestRecord& a, const RequestRecord& b) {
        return a.pages_per_split > b.pages_per_split;
    });
    int64_t items = 0;
    for (int32_t i = 0; i < n; ++i) {
        // ceil(N / pps) can be smaller than the S used to derive pps; keep only non-empty splits
        recs[i].num_splits = (recs[i].num_pages + recs[i].pages_per_split - 1) / recs[i].pages_per_split;
        recs[i].first_item = static_cast<int32_t>(items);
        items += static_cast<int64_t>(recs[i].num_splits) * geo.num_kv_heads;
        pos[recs[i].request] = i;
        if (items > INT32_MAX) return OSERVE_ERR_SHAPE;
    }
    records.swap(recs);
    position_of.swap(pos);
    batch = n;
    split_pages = c;
    num_items = static_cast<int32_t>(items);
    return OSERVE_OK;
}

}  // namespace oserve
