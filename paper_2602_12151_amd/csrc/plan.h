// Internal: host-side split plan shared by plan.cpp (sizing) and api.cpp (launch).
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "oserve.h"

namespace oserve {

// A run = consecutive splits of one request that all have the same size (the very last split of a
// request may be shorter).  One record per run, in launch order (largest splits first).  The device
// reads the records from pinned host memory and expands them into one ItemDesc per work item.
struct RunRecord {
    int32_t request;          // index b into q / block_table / context_lens / out
    int32_t first_item;       // index of the run's first work item; items are (split, kv head), kv head fastest
    int32_t num_splits;       // splits in this run
    int32_t pages_per_split;  // size of each of them
    int32_t page_begin;       // logical pages [page_begin, page_end) of the request belong to the run
    int32_t page_end;
    int32_t row_base;         // partial-result row group of the run's first split
    int32_t total_splits;     // splits of the whole request (1: the item writes `out` itself)
};
static_assert(sizeof(RunRecord) == 32, "record layout is part of the kernel interface");

// What one wavefront of the split kernel works on; written on the device from the run records.
struct ItemDesc {
    int32_t request_kvh;      // request | kv head << kKvHeadShift
    int32_t page_begin;       // logical pages [page_begin, page_end) of the request
    int32_t page_end;
    int32_t row;              // partial-result row group, or -1: the request has one split, write `out`
};
static_assert(sizeof(ItemDesc) == 16, "descriptor layout is part of the kernel interface");
constexpr int32_t kKvHeadShift = 20;       // requests < 2^20, kv heads < 2^11

struct RequestInfo {          // per request, in request order; read by the merge kernel
    int32_t split_base;       // first partial-result row group of the request
    int32_t num_splits;       // 0: the request is not a decode request of this launch (mixed batches)
    int32_t q_row;            // row of the request's query in q and out (= request index unless rows are packed)
    int32_t pad;
};
static_assert(sizeof(RequestInfo) == 16, "record layout is part of the kernel interface");

// The planner and the kernels work in tiles of kTileTokens tokens (one MFMA tile of keys); a page of
// the cache holds 1, 2 or 4 of them.  Wherever this code says "pages" of a split, a run or an item
// it counts tiles; the two coincide at the page size of 16.
constexpr int32_t kTileTokens = 16;

struct Geometry {
    int32_t num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq;
    int32_t group() const { return num_q_heads / num_kv_heads; }
    int32_t tiles_per_page() const { return page_size / kTileTokens; }
    int64_t max_tiles_per_seq() const { return static_cast<int64_t>(max_pages_per_seq) * tiles_per_page(); }
};

struct WorkspaceLayout {
    size_t req_info_off, items_off, partial_o_off, partial_ml_off, total;
};

// Split sizing.  In automatic mode the largest split C is one wavefront slot's fair share of the
// batch: (page-units of the batch) / (wavefront slots of the device), rounded up to a multiple of
// kSplitGranule pages, so the first, largest items fill every slot once and no slot ever holds two
// of them.  The end of every long request is cut into smaller splits taken from the ladder
// C, C/2, C/4, ... >= kSplitGranule (each rounded up to the granule); a request contributes at most
// kMaxRunsPerRequest runs.  Measured on the five workloads and modelled over scaled variants of
// them, whole multiples or fractions of the fair share other than 1 leave slots idle at the end
// (up to 20 % longer launches).
constexpr int32_t kSplitGranule = 12;
constexpr int32_t kMaxRunsPerRequest = 8;
constexpr int32_t kTailSlotsX16 = 6;        // tapered share = this/16 * slots * C page-units (see build())
constexpr int32_t kDefaultWaveSlots = 1024; // plans without a device: 256 compute units x 4 SIMDs

// Pure host logic (no HIP): everything the CPU tests exercise.
struct SplitPlan {
    Geometry geo{};
    int32_t capacity = 0;
    int32_t split_pages_user = 0;   // 0 = automatic
    int32_t wave_slots = kDefaultWaveSlots;   // wavefronts the split kernel keeps resident: compute units x SIMDs
    int32_t batch = 0;
    int32_t split_pages = 0;        // C actually used
    int32_t tail_q8 = 0;            // share of each long request that is tapered, in 1/256 (0: none)
    int32_t num_items = 0;
    int32_t num_row_groups = 0;     // sum of splits over all requests
    bool needs_merge = false;       // some request has more than one split
    std::vector<RunRecord> records;         // launch order
    std::vector<RequestInfo> req_info;      // request order
    std::vector<RunRecord> scratch_records; // build() works here, then swaps
    std::vector<RequestInfo> scratch_info;

    static oserve_status_t check_geometry(const Geometry& g, int32_t batch, int32_t capacity,
                                          int32_t split_tokens);
    void reserve();
    // q_lens == nullptr: every request is a decode request and its query row is its index.  Otherwise
    // request b brings q_lens[b] query rows packed after those of the requests before it, and only
    // the requests with q_lens[b] == 1 are planned here (the others get num_splits = 0 and no runs).
    oserve_status_t build(const int32_t* lens, int32_t n, const int32_t* q_lens = nullptr);
    WorkspaceLayout layout(int64_t items, int64_t row_groups, int32_t n) const;
    int64_t max_items() const;
    int64_t max_runs() const { return static_cast<int64_t>(capacity) * kMaxRunsPerRequest; }
};

}  // namespace oserve
