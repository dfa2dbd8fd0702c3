// Internal: kernel parameter blocks and launchers (kernels.hip), used by api.cpp.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "plan.h"

namespace oserve {

struct SplitParams {
    const ItemDesc* items;         // one per work item, launch order
    const RequestInfo* req_info;   // device copy, request order (read only where query rows are packed)
    const uint16_t* q;             // bf16 bits [B, Hq, D]
    const uint16_t* k_pages;       // bf16 bits [P, Hkv, page_size, D]
    const uint16_t* v_pages;
    const int32_t* block_table;    // [B, max_pages_per_seq]
    const int32_t* context_lens;   // [B]
    float* out;                    // [B, Hq, D]
    float* partial_o;              // [row_groups * Hq, D], un-normalised
    float* partial_ml;             // [row_groups * Hq, 2]: running max (log2 domain), normaliser
    float scale_log2e;             // scale * log2(e)
    int32_t num_q_heads, num_kv_heads, group, max_pages_per_seq;
    int32_t tile_shift;            // log2(page_size / 16): 16-token tiles per page
};

struct MergeParams {
    const RequestInfo* req_info;   // device copy, request order
    const float* partial_o;
    const float* partial_ml;
    float* out;
    int32_t num_q_heads;
};

struct ExpandParams {
    const RunRecord* records_host;    // pinned host memory as the device addresses it, 16-byte aligned
    int32_t num_runs;
    const RequestInfo* req_info_host; // pinned host memory, 16-byte aligned, readable up to a 16-byte boundary
    RequestInfo* req_info;            // workspace copy (whole 16-byte words are written)
    int32_t batch;
    ItemDesc* items;                  // workspace, one descriptor per work item
    int32_t num_kv_heads;
    uint32_t kv_heads_magic;          // floor(2^32 / num_kv_heads) + 1: (k * magic) >> 32 == k / num_kv_heads for k < 2^20
                                      // (unused when num_kv_heads == 1, where it does not fit 32 bits)
    const void* blob_host;            // further records copied as they are (pinned host memory, 16-byte aligned) ...
    void* blob;                       // ... into the workspace
    int32_t blob_words;               // their size in 16-byte words (0: none)
    int32_t* zero;                    // workspace words to clear (queue counters of the mixed kernel) ...
    int32_t zero_words;               // ... and their number (0: none)
};

// The events are attached to the kernel's own dispatch (no marker packets between the kernels):
// `done` completes when the expand kernel has finished; `start`/`stop`, if non-null, take the split
// kernel's begin and end timestamps.
hipError_t launch_expand(const ExpandParams& p, hipStream_t stream, hipEvent_t done);
hipError_t launch_split(const SplitParams& p, int head_dim, int num_items, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop);
hipError_t launch_merge(const MergeParams& p, int head_dim, int batch, hipStream_t stream);

// ---- chunked prefill (prefill.hip) ----
constexpr int kPrefillWaves = 4;        // wavefronts that share a prefill item (one per SIMD; two workgroups per compute unit)
constexpr int kPrefillColTiles = 2;     // 16-column score tiles per wavefront
constexpr int kPrefillMacroKeys = 64;   // keys staged in LDS per barrier
// query tokens of one work item for a GQA group of 1 << group_shift heads
inline int prefill_block_tokens(int group_shift) { return kPrefillWaves * ((16 * kPrefillColTiles) >> group_shift); }

// One workgroup's work: a block of query tokens of one request against one kv head.
struct PrefillItem {
    int32_t request;       // index into block_table rows
    int32_t kv_head;
    int32_t q_begin;       // first query token of the block, counted within the request
    int32_t q_row0;        // packed row (in q / out) of the request's query token 0
    int32_t context_len;   // L: cached tokens of the request, the new ones included
    int32_t q_len;         // n: new query tokens of the request
    int32_t pad[2];
};
static_assert(sizeof(PrefillItem) == 32, "item layout is part of the kernel interface");

struct PrefillParams {
    const PrefillItem* items;      // pinned host memory as the device addresses it, launch order
    const uint16_t* q;             // bf16 bits [sum n, Hq, D], requests packed
    const uint16_t* k_pages;       // bf16 bits [P, Hkv, page_size, D]
    const uint16_t* v_pages;
    const int32_t* block_table;    // [B, max_pages_per_seq]
    float* out;                    // [sum n, Hq, D]
    float scale_log2e;
    int32_t num_q_heads, num_kv_heads, group, group_shift, max_pages_per_seq, tile_shift;
};

hipError_t launch_prefill(const PrefillParams& p, int head_dim, int num_items, hipStream_t stream,
                          hipEvent_t start, hipEvent_t stop);

// ---- mixed prefill + decode batches (mixed.hip) ----
constexpr int kMaxQueueXcds = 16;   // prefill queues (one per XCD) the mixed kernel can address

struct MixedParams {
    SplitParams decode;       // items, req_info and partials in the workspace; q / out rows packed
    PrefillParams prefill;    // items in the workspace: XCD 0's queue, then XCD 1's, ...
    int32_t* queue_next;      // workspace, [kMaxQueueXcds + 1], zero at kernel start: next entry of each XCD's
                              // prefill queue, then (index kMaxQueueXcds) of the decode queue
    int32_t prefill_queue_first[kMaxQueueXcds];   // index of the first prefill item of each XCD's queue ...
    int32_t prefill_queue_size[kMaxQueueXcds];    // ... and their number
    int32_t num_xcds;
    int32_t num_decode_items; // the decode queue is the decode items in launch order
};

// num_workgroups: two per compute unit (each lasts for the whole launch and takes work from the queues).
hipError_t launch_mixed(const MixedParams& p, int head_dim, int num_workgroups, hipStream_t stream,
                        hipEvent_t start, hipEvent_t stop);

// ---- KV-block migration copies (migrate.hip) ----
struct MigrateParams {
    const void* k_src;            // gather: page pool; scatter: staging chunk
    const void* v_src;
    void* k_dst;                  // gather: staging chunk; scatter: page pool
    void* v_dst;
    const int32_t* block_table;   // names the pool pages (source table for gather, target table for scatter)
    int32_t table_stride;         // entries per table row
    const int32_t* page_refs;     // [num_pages][4] per staging page: source table row of its request, index of its
                                  // request, page index within the request, 0
    int32_t use_source_rows;      // table row of a page: its request's source row (1) or its request's index (0)
    int64_t num_pages;            // staging pages
    int32_t pool_heads;           // kv heads per page in the pool
    int32_t head_begin;           // first pool head of the copied range
    int32_t num_heads;            // heads copied (= heads per page of the staging chunk)
    int32_t unit_chunks;          // 16-byte chunks per (page, head): page_size * head_dim * 2 / 16
};

hipError_t launch_kv_migrate(const MigrateParams& p, bool gather, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop);

}  // namespace oserve
