// Host-side work list of the chunked-prefill kernel: which workgroup computes which block of query
// tokens against which kv head, and in which launch order.
#include "prefill_plan.h"

#include <algorithm>

namespace oserve {

oserve_status_t PrefillWorkList::check_geometry(const Geometry& g, int32_t batch, int32_t capacity,
                                                int64_t max_query_tokens) {
    const oserve_status_t st = SplitPlan::check_geometry(g, batch, capacity, 0);
    if (st != OSERVE_OK) return st;
    // (head_dim 64 or 128 and any group size up to 16, which the kernel pads to a power of two: what the
    // decode plan accepts)
    if (max_query_tokens < 1 || max_query_tokens > (1ll << 28)) return OSERVE_ERR_SHAPE;
    return OSERVE_OK;
}

void PrefillWorkList::reserve() {
    const size_t n = static_cast<size_t>(max_items());
    items.reserve(n);
    scratch.reserve(n);
    for (int x = 0; x < xcds; ++x) per_xcd[x].reserve(n);
    groups.reserve(static_cast<size_t>(capacity) * geo.num_kv_heads);
    row0.reserve(static_cast<size_t>(capacity) + 1);
}

oserve_status_t PrefillWorkList::build(const int32_t* lens, const int32_t* qlens, int32_t n, bool skip_single_token) {
    if (!lens || !qlens) return OSERVE_ERR_NULL;
    if (n < 1 || n > capacity) return OSERVE_ERR_PLAN_MISMATCH;
    const int64_t max_len = static_cast<int64_t>(geo.max_pages_per_seq) * geo.page_size;
    int64_t total_q = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (lens[b] < 1 || lens[b] > max_len || qlens[b] < 1 || qlens[b] > lens[b]) return OSERVE_ERR_CONTEXT_LEN;
        total_q += qlens[b];
    }
    if (total_q > max_query_tokens) return OSERVE_ERR_PLAN_MISMATCH;
    const int32_t qb = block_tokens();
    const int32_t hkv = geo.num_kv_heads;
    // Groups = (request, kv head): all query blocks of a group read the same K/V.  Workgroups go to
    // the device's XCDs round-robin by index, and every XCD has its own L2, so the blocks of a group
    // are placed at indices that are equal modulo the XCD count: they then run side by side on one
    // XCD and its L2 serves the K/V tiles that the first of them fetched.  Groups are dealt to the
    // XCDs heaviest first, each to the XCD with the least work so far; inside a group the blocks
    // with the most keys come first.
    groups.clear();
    for (int32_t b = 0; b < n; ++b) {
        if (skip_single_token && qlens[b] == 1) continue;
        int64_t work = 0;
        for (int32_t q0 = 0; q0 < qlens[b]; q0 += qb)
            work += lens[b] - qlens[b] + std::min(q0 + qb, qlens[b]);
        for (int32_t j = 0; j < hkv; ++j) groups.push_back(Group{b, j, work});
    }
    std::stable_sort(groups.begin(), groups.end(), [](const Group& a, const Group& c) { return a.work > c.work; });
    row0.assign(static_cast<size_t>(n) + 1, 0);
    for (int32_t b = 0; b < n; ++b) row0[b + 1] = row0[b] + qlens[b];
    int64_t load[kMaxXcds] = {};
    for (int x = 0; x < xcds; ++x) per_xcd[x].clear();
    for (const Group& g : groups) {
        int best = 0;
        for (int x = 1; x < xcds; ++x)
            if (load[x] < load[best]) best = x;
        load[best] += g.work;
        const int32_t b = g.request;
        const int32_t blocks = (qlens[b] + qb - 1) / qb;
        for (int32_t k = blocks - 1; k >= 0; --k)     // last blocks see the most keys
            per_xcd[best].push_back(PrefillItem{b, g.kv_head, k * qb, static_cast<int32_t>(row0[b]), lens[b], qlens[b], {0, 0}});
    }
    // interleave: position xcds * k + x takes the k-th item of XCD x's list; exhausted lists are skipped
    scratch.clear();
    size_t cursor[kMaxXcds] = {};
    for (bool any = true; any;) {
        any = false;
        for (int x = 0; x < xcds; ++x)
            if (cursor[x] < per_xcd[x].size()) {
                scratch.push_back(per_xcd[x][cursor[x]++]);
                any = true;
            }
    }
    items.swap(scratch);
    batch = n;
    query_tokens = total_q;
    return OSERVE_OK;
}

}  // namespace oserve
