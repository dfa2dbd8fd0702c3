// Host-side planning: sizes the per-request sequence splits of a mixed-length batch so that short
// and long requests fill the device together (the spatially heterogeneous batch of paper section
// 1 (i) / section 2).
#include "plan.h"

#include <algorithm>
#include <cstdlib>

namespace oserve {

oserve_status_t SplitPlan::check_geometry(const Geometry& g, int32_t batch, int32_t capacity,
                                          int32_t split_tokens) {
    if (g.num_q_heads < 1 || g.num_kv_heads < 1 || g.num_q_heads % g.num_kv_heads != 0)
        return OSERVE_ERR_SHAPE;
    if (g.group() > 16 || g.num_kv_heads >= (1 << (31 - kKvHeadShift))) return OSERVE_ERR_SHAPE;
    if (g.head_dim != 64 && g.head_dim != 128) return OSERVE_ERR_SHAPE;
    if (g.page_size != 16 && g.page_size != 32 && g.page_size != 64) return OSERVE_ERR_SHAPE;
    if (g.max_pages_per_seq < 1 || g.max_tiles_per_seq() > (1 << 26)) return OSERVE_ERR_SHAPE;
    if (batch < 1 || capacity < batch || capacity > (1 << kKvHeadShift)) return OSERVE_ERR_SHAPE;
    if (split_tokens < 0 || split_tokens % g.page_size != 0) return OSERVE_ERR_SHAPE;
    return OSERVE_OK;
}

void SplitPlan::reserve() {
    records.reserve(static_cast<size_t>(max_runs()));
    scratch_records.reserve(static_cast<size_t>(max_runs()));
    req_info.reserve(static_cast<size_t>(capacity));
    scratch_info.reserve(static_cast<size_t>(capacity));
}

int64_t SplitPlan::max_items() const {
    // the smallest split the plan can choose bounds the item count from above
    const int64_t c_min = split_pages_user > 0 ? split_pages_user : kSplitGranule;
    const int64_t per_req = (geo.max_tiles_per_seq() + c_min - 1) / c_min + kMaxRunsPerRequest;
    return per_req * capacity * geo.num_kv_heads;
}

WorkspaceLayout SplitPlan::layout(int64_t items, int64_t row_groups, int32_t n) const {
    auto align = [](size_t x) { return (x + 255) & ~static_cast<size_t>(255); };
    WorkspaceLayout w{};
    w.req_info_off = 0;
    w.items_off = align(static_cast<size_t>(n) * sizeof(RequestInfo) + 16);  // copied in whole 16-byte words
    w.partial_o_off = w.items_off + align(static_cast<size_t>(items) * sizeof(ItemDesc));
    const size_t rows = static_cast<size_t>(row_groups) * geo.num_q_heads;
    w.partial_ml_off = w.partial_o_off + align(rows * geo.head_dim * sizeof(float));
    w.total = w.partial_ml_off + align(rows * 2 * sizeof(float));
    return w;
}

namespace {

inline int32_t round_up(int32_t x, int32_t g) { return (x + g - 1) / g * g; }

}  // namespace

oserve_status_t SplitPlan::build(const int32_t* lens, int32_t n, const int32_t* q_lens) {
    if (!lens) return OSERVE_ERR_NULL;
    if (n < 1 || n > capacity) return OSERVE_ERR_PLAN_MISMATCH;
    const int64_t max_len = static_cast<int64_t>(geo.max_pages_per_seq) * geo.page_size;
    int64_t total_pages = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (lens[b] < 1 || lens[b] > max_len) return OSERVE_ERR_CONTEXT_LEN;
        if (q_lens && (q_lens[b] < 1 || q_lens[b] > lens[b])) return OSERVE_ERR_CONTEXT_LEN;
        if (!q_lens || q_lens[b] == 1) total_pages += (lens[b] + kTileTokens - 1) / kTileTokens;
    }

    // ---- size of the largest split, and the share of each long request that is tapered ----
    int32_t c = split_pages_user;
    int32_t taper_q8 = 0;
    if (c == 0) {
        const int64_t slots = std::max<int64_t>(1, wave_slots);
        const int64_t units = total_pages * geo.num_kv_heads;
        const int64_t want = std::min<int64_t>(geo.max_tiles_per_seq(), std::max<int64_t>(kSplitGranule, (units + slots - 1) / slots));
        c = round_up(static_cast<int32_t>(want), kSplitGranule);
        // Work is handed out evenly only while an item is no longer than what is left per slot.
        // Full-size items therefore stop when about slots * C page-units are left, and from there
        // the splits shrink with what remains: that last share of every long request is tapered.
        const int64_t q8 = units > 0 ? (16 * kTailSlotsX16 * slots * c + units - 1) / units : 0;
        taper_q8 = static_cast<int32_t>(std::min<int64_t>(192, q8));
    }
    // ladder of split sizes for the tapered part
    int32_t ladder[kMaxRunsPerRequest];
    int32_t n_ladder = 0;
    for (int32_t k = 0; n_ladder < kMaxRunsPerRequest - 1; ++k) {
        const int32_t v = std::max(kSplitGranule, round_up(c >> k, kSplitGranule));
        if (n_ladder > 0 && v >= ladder[n_ladder - 1]) break;
        ladder[n_ladder++] = std::min(v, c);
        if (v == kSplitGranule) break;
    }

    std::vector<RunRecord>& recs = scratch_records;   // reserved to the bound: no allocation here
    std::vector<RequestInfo>& info = scratch_info;
    recs.clear();
    info.resize(static_cast<size_t>(n));
    int64_t row_groups = 0;
    int64_t q_row = 0;
    bool any_split = false;
    for (int32_t b = 0; b < n; ++b) {
        if (q_row > (1ll << 30)) return OSERVE_ERR_SHAPE;
        if (q_lens && q_lens[b] != 1) {      // not a decode request: no runs
            info[b] = RequestInfo{static_cast<int32_t>(row_groups), 0, static_cast<int32_t>(q_row), 0};
            q_row += q_lens[b];
            continue;
        }
        const int32_t pages = (lens[b] + kTileTokens - 1) / kTileTokens;
        const size_t first_rec = recs.size();
        int32_t splits = 0;
        auto add_run = [&](int32_t begin, int32_t count, int32_t pps, int32_t end) {
            recs.push_back(RunRecord{b, 0, count, pps, begin, end, static_cast<int32_t>(row_groups) + splits, 0});
            splits += count;
        };
        if (pages <= c) {
            add_run(0, 1, pages, pages);
        } else if (taper_q8 == 0) {
            // near-equal splits: S = ceil(N / C) splits of ceil(N / S) pages (S recomputed so none is empty)
            const int32_t s0 = (pages + c - 1) / c;
            const int32_t pps = (pages + s0 - 1) / s0;
            add_run(0, (pages + pps - 1) / pps, pps, pages);
        } else {
            const int32_t tail = std::max<int32_t>(c, static_cast<int32_t>((static_cast<int64_t>(pages) * taper_q8) >> 8));
            int32_t pos = 0;
            // full-size splits while more than the tail is left
            const int32_t n_full = pages > tail ? (pages - tail + c - 1) / c : 0;
            if (n_full > 0) {
                add_run(0, n_full, c, std::min(pages, n_full * c));
                pos = std::min(pages, n_full * c);
            }
            // tapered part: each ladder size is used while the proportional size still reaches it
            for (int32_t k = 0; k < n_ladder && pos < pages; ++k) {
                const int32_t size = ladder[k];
                const bool last_rung = k == n_ladder - 1;
                // proportional size at `remaining` is remaining * C / tail; rung k serves remaining
                // down to the point where that falls below the next rung
                const int32_t next = last_rung ? 0 : ladder[k + 1];
                const int32_t stop_remaining = last_rung ? 0 : static_cast<int32_t>((static_cast<int64_t>(next) * tail) / c);
                const int32_t remaining = pages - pos;
                if (remaining <= stop_remaining) continue;
                const int32_t span = remaining - stop_remaining;
                // whole splits only, except on the last rung, which also takes the ragged end
                int32_t count = last_rung ? (span + size - 1) / size : span / size;
                if (count == 0) continue;
                const int32_t end = std::min(pages, pos + count * size);
                add_run(pos, count, size, end);
                pos = end;
            }
        }
        for (size_t i = first_rec; i < recs.size(); ++i) recs[i].total_splits = splits;
        info[b] = RequestInfo{static_cast<int32_t>(row_groups), splits, static_cast<int32_t>(q_lens ? q_row : b), 0};
        q_row += 1;
        row_groups += splits;
        any_split = any_split || splits > 1;
        if (recs.size() > static_cast<size_t>(max_runs())) return OSERVE_ERR_SHAPE;
    }
    // largest splits first; ties keep request order, so the launch order is deterministic
    std::stable_sort(recs.begin(), recs.end(), [](const RunRecord& a, const RunRecord& b) {
        return a.pages_per_split > b.pages_per_split;
    });
    int64_t items = 0;
    for (RunRecord& r : recs) {
        r.first_item = static_cast<int32_t>(items);
        const int64_t run_items = static_cast<int64_t>(r.num_splits) * geo.num_kv_heads;
        // per-run bound: the device splits an item index into (split, kv head) with a 32-bit
        // multiply-high that is exact below 2^20
        if (run_items > (1 << 20)) return OSERVE_ERR_SHAPE;
        items += run_items;
        if (items > (1 << 30)) return OSERVE_ERR_SHAPE;
    }
    if (row_groups * geo.num_q_heads > (1 << 30)) return OSERVE_ERR_SHAPE;
    records.swap(recs);
    req_info.swap(info);
    batch = n;
    split_pages = c;
    tail_q8 = taper_q8;
    num_items = static_cast<int32_t>(items);
    num_row_groups = static_cast<int32_t>(row_groups);
    needs_merge = any_split;
    return OSERVE_OK;
}

}  // namespace oserve
