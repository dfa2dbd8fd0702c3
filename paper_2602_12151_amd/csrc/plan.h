// Internal: host-side split plan shared by plan.cpp (sizing) and api.hip (launch).
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "oserve.h"

namespace oserve {

// One record per request, in launch order (longest split first).  Uploaded to
// the front of the workspace; the kernels find their request by binary search
// over first_item.
struct RequestRecord {
    int32_t request;          // index b into q / block_table / context_lens / out
    int32_t first_item;       // index of this request's first work item
    int32_t num_splits;       // S_b
    int32_t pages_per_split;  // ceil(N_b / S_b)
    int32_t num_pages;        // N_b = ceil(L_b / page_size)
    int32_t pad[3];
};
static_assert(sizeof(RequestRecord) == 32, "record layout is part of the kernel interface");

struct Geometry {
    int32_t num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq;
    int32_t group() const { return num_q_heads / num_kv_heads; }
};

struct WorkspaceLayout {
    size_t records_off, partial_o_off, partial_ml_off, total;
};

// Pure host logic (no HIP): everything the CPU tests exercise.
struct SplitPlan {
    Geometry geo{};
    int32_t capacity = 0;
    int32_t split_pages_user = 0;   // 0 = automatic
    int32_t num_cus = 256;
    int32_t batch = 0;
    int32_t split_pages = 0;        // C actually used
    int32_t num_items = 0;
    std::vector<RequestRecord> records;     // launch order, size batch
    std::vector<int32_t> position_of;       // request -> index into records
    std::vector<RequestRecord> scratch_records;   // build() works here, then swaps
    std::vector<int32_t> scratch_position;

    static oserve_status_t check_geometry(const Geometry& g, int32_t batch, int32_t capacity,
                                          int32_t split_tokens);
    oserve_status_t build(const int32_t* lens, int32_t n);
    WorkspaceLayout layout(int64_t items, int32_t n) const;
    int64_t max_items() const;
};

// Target number of work items: waves the device keeps resident times an
// oversubscription factor, so the tail of the launch is short.
constexpr int32_t kWavesPerCu = 8;
constexpr int32_t kOversubscribe = 4;
constexpr int32_t kMinSplitPages = 8;

}  // namespace oserve
