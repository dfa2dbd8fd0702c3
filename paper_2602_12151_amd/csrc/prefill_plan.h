// Internal: host-side work list of the chunked-prefill kernel (blocks of query tokens x kv heads),
// shared by the prefill plan (api_prefill.cpp) and the mixed prefill + decode plan (api_mixed.cpp).
#pragma once
#include <cstdint>
#include <vector>

#include "kernels.h"
#include "oserve.h"
#include "plan.h"

namespace oserve {

constexpr int kMaxXcds = 16;

// Pure host logic (no HIP).
struct PrefillWorkList {
    Geometry geo{};
    int32_t capacity = 0;            // largest batch
    int64_t max_query_tokens = 0;    // largest sum of query lengths
    int32_t xcds = 8;                // accelerator dies of the device, each with its own L2 (8 without a device)
    int32_t batch = 0;
    int64_t query_tokens = 0;        // sum of the query lengths of all requests of the batch
    std::vector<PrefillItem> items;              // launch order: position xcds * k + x = k-th item of XCD x's list
    std::vector<PrefillItem> per_xcd[kMaxXcds];  // the same items, per XCD
    std::vector<PrefillItem> scratch;
    struct Group { int32_t request, kv_head; int64_t work; };
    std::vector<Group> groups;
    std::vector<int64_t> row0;

    static oserve_status_t check_geometry(const Geometry& g, int32_t batch, int32_t capacity, int64_t max_query_tokens);
    int32_t group_shift() const {
        int32_t s = 0;
        while ((1 << s) < geo.group()) ++s;
        return s;
    }
    int32_t block_tokens() const { return prefill_block_tokens(group_shift()); }   // query tokens per workgroup
    int64_t max_items() const { return (max_query_tokens / block_tokens() + capacity) * geo.num_kv_heads; }
    void reserve();
    // skip_single_token: requests that bring one query token get no items (a mixed batch serves
    // them as decode requests); their rows still count in the packing of q and out.
    oserve_status_t build(const int32_t* lens, const int32_t* qlens, int32_t n, bool skip_single_token);
    // key tiles of kPrefillMacroKeys keys that item `it` walks over
    static int32_t macro_steps(const PrefillItem& it, int32_t block_tokens) {
        const int32_t last_tok = (it.q_begin + block_tokens < it.q_len ? it.q_begin + block_tokens : it.q_len) - 1;
        return (it.context_len - it.q_len + last_tok) / kPrefillMacroKeys + 1;
    }
};

}  // namespace oserve
