// Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the library's host-only code
// and of the oracle (CPU only; built and run by tests/test_sanitizers.py).  It drives the split planner,
// the prefill work list and the switch / assignment planners over seeded random inputs and checks the
// invariants their callers rely on; any sanitizer report or failed check ends the process with an error.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "oserve.h"
#include "plan.h"
#include "prefill_plan.h"

extern "C" int oserve_oracle_paged_decode_attn(const uint16_t* q, int64_t q_stride_b, int64_t q_stride_h,
                                               const uint16_t* k_pages, const uint16_t* v_pages, int64_t num_pages,
                                               int64_t kv_stride_page, int64_t kv_stride_head, int64_t kv_stride_tok,
                                               const int32_t* block_table, int64_t bt_stride, const int32_t* context_lens,
                                               int32_t batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                                               int32_t page_size, float scale, double* out, double* lse);

namespace {

uint64_t state = 0x9E3779B97F4A7C15ull;
uint64_t next_u64() {   // splitmix64
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
int64_t uniform(int64_t lo, int64_t hi) { return lo + static_cast<int64_t>(next_u64() % static_cast<uint64_t>(hi - lo + 1)); }

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

// every tile of every planned request is covered by exactly one split; sizes and bounds hold
void check_split_plan(const oserve::SplitPlan& pl, const std::vector<int32_t>& lens, const int32_t* qlens) {
    const int32_t n = static_cast<int32_t>(lens.size());
    std::vector<std::vector<int32_t>> covered(n);
    for (int32_t b = 0; b < n; ++b) covered[b].assign((lens[b] + 15) / 16, 0);
    int64_t items = 0;
    int32_t prev = INT32_MAX;
    for (const oserve::RunRecord& r : pl.records) {
        CHECK(r.request >= 0 && r.request < n);
        CHECK(!qlens || qlens[r.request] == 1);
        CHECK(r.first_item == items);
        CHECK(r.num_splits >= 1 && r.pages_per_split >= 1 && r.pages_per_split <= pl.split_pages);
        CHECK(r.pages_per_split <= prev);
        prev = r.pages_per_split;
        CHECK(0 <= r.page_begin && r.page_begin < r.page_end && r.page_end <= static_cast<int32_t>(covered[r.request].size()));
        const int32_t span = r.page_end - r.page_begin;
        CHECK((r.num_splits - 1) * r.pages_per_split < span && span <= r.num_splits * r.pages_per_split);
        for (int32_t p = r.page_begin; p < r.page_end; ++p) covered[r.request][p] += 1;
        CHECK(r.total_splits == pl.req_info[r.request].num_splits);
        CHECK(r.row_base >= pl.req_info[r.request].split_base &&
              r.row_base + r.num_splits <= pl.req_info[r.request].split_base + r.total_splits);
        items += static_cast<int64_t>(r.num_splits) * pl.geo.num_kv_heads;
    }
    CHECK(items == pl.num_items && items <= pl.max_items());
    CHECK(static_cast<int64_t>(pl.records.size()) <= pl.max_runs());
    int64_t rows = 0, q_row = 0;
    for (int32_t b = 0; b < n; ++b) {
        const bool planned = !qlens || qlens[b] == 1;
        for (int32_t c : covered[b]) CHECK(c == (planned ? 1 : 0));
        CHECK(pl.req_info[b].split_base == rows);
        CHECK(planned ? pl.req_info[b].num_splits >= 1 : pl.req_info[b].num_splits == 0);
        CHECK(pl.req_info[b].q_row == (qlens ? q_row : b));
        rows += pl.req_info[b].num_splits;
        q_row += qlens ? qlens[b] : 1;
    }
    CHECK(rows == pl.num_row_groups);
    const oserve::WorkspaceLayout now = pl.layout(pl.num_items, pl.num_row_groups, pl.batch);
    const oserve::WorkspaceLayout most = pl.layout(pl.max_items(), pl.max_items() / pl.geo.num_kv_heads, pl.capacity);
    CHECK(now.total <= most.total);
}

void fuzz_split_plans(int rounds) {
    static const int32_t heads[][2] = {{32, 8}, {16, 2}, {8, 8}, {16, 1}, {24, 3}, {7, 7}, {64, 8}};
    for (int it = 0; it < rounds; ++it) {
        const int32_t* h = heads[uniform(0, 6)];
        const int32_t page = 16 << uniform(0, 2);
        const int32_t max_pages = static_cast<int32_t>(uniform(1, it % 7 == 0 ? 9000 : 600));
        oserve::SplitPlan pl;
        pl.geo = oserve::Geometry{h[0], h[1], uniform(0, 1) ? 128 : 64, page, max_pages};
        pl.capacity = static_cast<int32_t>(uniform(1, 96));
        const int32_t explicit_pages = uniform(0, 3) == 0 ? static_cast<int32_t>(uniform(1, 64)) * (page / 16) : 0;
        pl.split_pages_user = explicit_pages;
        pl.wave_slots = static_cast<int32_t>(uniform(1, 2048));
        CHECK(oserve::SplitPlan::check_geometry(pl.geo, 1, pl.capacity, explicit_pages * 16) == OSERVE_OK);
        pl.reserve();
        for (int update = 0; update < 3; ++update) {
            const int32_t n = static_cast<int32_t>(uniform(1, pl.capacity));
            std::vector<int32_t> lens(n), qlens(n);
            const int64_t max_len = static_cast<int64_t>(max_pages) * page;
            for (int32_t b = 0; b < n; ++b) {
                lens[b] = static_cast<int32_t>(uniform(0, 3) ? uniform(1, max_len) : uniform(1, std::min<int64_t>(max_len, 300)));
                qlens[b] = uniform(0, 2) ? 1 : static_cast<int32_t>(uniform(1, lens[b]));
            }
            const bool mixed = uniform(0, 1);
            CHECK(pl.build(lens.data(), n, mixed ? qlens.data() : nullptr) == OSERVE_OK);
            check_split_plan(pl, lens, mixed ? qlens.data() : nullptr);
            // refused inputs leave the plan as it was
            const int32_t items_before = pl.num_items;
            std::vector<int32_t> bad = lens;
            bad[uniform(0, n - 1)] = uniform(0, 1) ? 0 : static_cast<int32_t>(std::min<int64_t>(max_len + 1, INT32_MAX));
            CHECK(pl.build(bad.data(), n) == OSERVE_ERR_CONTEXT_LEN);
            CHECK(pl.num_items == items_before);
        }
    }
}

void fuzz_prefill_lists(int rounds) {
    static const int32_t heads[][2] = {{32, 8}, {16, 2}, {8, 8}, {16, 1}, {4, 2}, {12, 4}, {6, 2}, {14, 2}};
    for (int it = 0; it < rounds; ++it) {
        const int32_t* h = heads[uniform(0, 7)];
        oserve::PrefillWorkList pl;
        pl.geo = oserve::Geometry{h[0], h[1], uniform(0, 1) ? 128 : 64, 16 << uniform(0, 2), static_cast<int32_t>(uniform(1, 300))};
        pl.capacity = static_cast<int32_t>(uniform(1, 40));
        pl.max_query_tokens = uniform(1, 20000);
        pl.xcds = static_cast<int32_t>(uniform(1, oserve::kMaxXcds));
        CHECK(oserve::PrefillWorkList::check_geometry(pl.geo, 1, pl.capacity, pl.max_query_tokens) == OSERVE_OK);
        pl.reserve();
        const int32_t n = static_cast<int32_t>(uniform(1, pl.capacity));
        std::vector<int32_t> lens(n), qlens(n);
        const int64_t max_len = static_cast<int64_t>(pl.geo.max_pages_per_seq) * pl.geo.page_size;
        int64_t total_q = 0;
        for (int32_t b = 0; b < n; ++b) {
            lens[b] = static_cast<int32_t>(uniform(1, max_len));
            qlens[b] = uniform(0, 1) ? 1 : static_cast<int32_t>(uniform(1, std::min<int64_t>(lens[b], 700)));
            total_q += qlens[b];
        }
        const bool skip = uniform(0, 1);
        const oserve_status_t st = pl.build(lens.data(), qlens.data(), n, skip);
        if (total_q > pl.max_query_tokens) { CHECK(st == OSERVE_ERR_PLAN_MISMATCH); continue; }
        CHECK(st == OSERVE_OK);
        const int32_t qb = pl.block_tokens();
        int64_t expect = 0, row = 0;
        std::vector<int64_t> row0(n);
        for (int32_t b = 0; b < n; ++b) {
            row0[b] = row;
            row += qlens[b];
            if (!(skip && qlens[b] == 1)) expect += static_cast<int64_t>((qlens[b] + qb - 1) / qb) * pl.geo.num_kv_heads;
        }
        CHECK(static_cast<int64_t>(pl.items.size()) == expect && expect <= pl.max_items());
        size_t in_lists = 0;
        for (int x = 0; x < pl.xcds; ++x) in_lists += pl.per_xcd[x].size();
        CHECK(in_lists == pl.items.size());
        for (const oserve::PrefillItem& i : pl.items) {
            CHECK(i.request >= 0 && i.request < n && i.kv_head >= 0 && i.kv_head < pl.geo.num_kv_heads);
            CHECK(i.q_len == qlens[i.request] && i.context_len == lens[i.request] && i.q_row0 == row0[i.request]);
            CHECK(i.q_begin % qb == 0 && i.q_begin < i.q_len);
            CHECK(oserve::PrefillWorkList::macro_steps(i, qb) >= 1);
        }
    }
}

void fuzz_planners(int rounds) {
    for (int it = 0; it < rounds; ++it) {
        // greedy switch plan
        const int32_t devices = static_cast<int32_t>(uniform(1, 12)), shards = static_cast<int32_t>(uniform(0, 10));
        std::vector<int32_t> machine(devices), so(shards + 1, 0), to(shards + 1, 0), sd, td;
        std::vector<int64_t> vol;
        for (int32_t& m : machine) m = static_cast<int32_t>(uniform(0, 3));
        for (int32_t m = 0; m < shards; ++m) {
            const int64_t ns = uniform(1, devices), nt = uniform(0, devices);
            for (int64_t k = 0; k < ns; ++k) sd.push_back(static_cast<int32_t>(uniform(0, devices - 1)));
            for (int64_t k = 0; k < nt; ++k) { td.push_back(static_cast<int32_t>(uniform(0, devices - 1))); vol.push_back(uniform(0, 1000)); }
            so[m + 1] = static_cast<int32_t>(sd.size());
            to[m + 1] = static_cast<int32_t>(td.size());
        }
        std::vector<int32_t> chosen(td.size() + 1, -7);
        std::vector<int64_t> load(static_cast<size_t>(devices) * devices, 0);
        sd.push_back(0); td.push_back(0); vol.push_back(0);   // never read: the offsets end before them
        CHECK(oserve_switch_plan(devices, machine.data(), shards, so.data(), sd.data(), to.data(), td.data(), vol.data(),
                                 chosen.data(), load.data()) == OSERVE_OK);
        for (int32_t m = 0; m < shards; ++m)
            for (int32_t i = to[m]; i < to[m + 1]; ++i) CHECK(chosen[i] >= -1 && chosen[i] < devices);
        CHECK(chosen[td.size() - 1] == -7);
        // capacity normalisation and workload assignment
        const int32_t reps = static_cast<int32_t>(uniform(1, 5)), types = static_cast<int32_t>(uniform(1, 5));
        std::vector<int64_t> cap(static_cast<size_t>(reps) * types), units(types);
        std::vector<double> arrivals(types), x(cap.size()), edge(cap.size());
        for (int64_t& c : cap) c = uniform(0, 4) ? uniform(1, 60) : 0;
        for (double& a : arrivals) a = static_cast<double>(uniform(0, 200));
        for (double& e : edge) e = static_cast<double>(uniform(0, 100));
        int64_t common = 0;
        CHECK(oserve_capacity_normalise(cap.data(), types, &common, units.data()) == OSERVE_OK);
        for (int32_t j = 0; j < types; ++j) CHECK(cap[j] == 0 ? units[j] == 0 : units[j] * cap[j] == common);
        double total = -1.0;
        CHECK(oserve_assign_workload(reps, types, arrivals.data(), cap.data(), uniform(0, 1) ? edge.data() : nullptr, x.data(),
                                     &total) == OSERVE_OK);
        double sum = 0.0;
        for (double v : x) { CHECK(v >= -1e-9); sum += v; }
        CHECK(total >= -1e-9 && sum <= total + 1e-6 && total <= sum + 1e-6);
    }
}

void run_oracle_once() {
    // a tiny paged batch with a ragged last page, to put the oracle's indexing under the sanitizers
    const int32_t B = 3, Hq = 4, Hkv = 2, D = 8, page = 16, pages = 7, width = 3;
    std::vector<uint16_t> q(B * Hq * D), k(pages * Hkv * page * D), v(k.size());
    for (uint16_t& e : q) e = static_cast<uint16_t>(0x3C00 + (next_u64() & 0x3FF));
    for (uint16_t& e : k) e = static_cast<uint16_t>(0x3C00 + (next_u64() & 0x3FF));
    for (uint16_t& e : v) e = static_cast<uint16_t>(0x3C00 + (next_u64() & 0x3FF));
    const int32_t bt[B * width] = {6, 0, -1, 2, -1, -1, 5, 1, 3};
    const int32_t lens[B] = {17, 1, 48};
    std::vector<double> out(B * Hq * D), lse(B * Hq);
    CHECK(oserve_oracle_paged_decode_attn(q.data(), Hq * D, D, k.data(), v.data(), pages, Hkv * page * D, page * D, D, bt, width,
                                          lens, B, Hq, Hkv, D, page, 0.35f, out.data(), lse.data()) == 0);
    for (double e : out) CHECK(e == e);
}

}  // namespace

int main(int argc, char** argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 1500;
    fuzz_split_plans(rounds);
    fuzz_prefill_lists(rounds);
    fuzz_planners(rounds);
    run_oracle_once();
    std::printf("ok: %d rounds each of split plans, prefill work lists and planners\n", rounds);
    return 0;
}
