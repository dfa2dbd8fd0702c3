// Internal: kernel parameter blocks and launchers (kernels.hip), used by api.cpp.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "plan.h"

namespace oserve {

struct SplitParams {
    const RunRecord* records;      // device copy, launch order
    int32_t num_runs;
    const uint16_t* q;             // bf16 bits [B, Hq, D]
    const uint16_t* k_pages;       // bf16 bits [P, Hkv, 16, D]
    const uint16_t* v_pages;
    const int32_t* block_table;    // [B, max_pages_per_seq]
    const int32_t* context_lens;   // [B]
    float* out;                    // [B, Hq, D]
    float* partial_o;              // [row_groups * Hq, D], un-normalised
    float* partial_ml;             // [row_groups * Hq, 2]: running max (log2 domain), normaliser
    float scale_log2e;             // scale * log2(e)
    int32_t num_q_heads, num_kv_heads, group, max_pages_per_seq;
};

struct MergeParams {
    const RequestInfo* req_info;   // device copy, request order
    const float* partial_o;
    const float* partial_ml;
    float* out;
    int32_t num_q_heads;
};

// src_host: pinned host memory as the device addresses it; copies `bytes` (rounded up to 16)
hipError_t launch_upload(const void* src_host, void* dst, size_t bytes, hipStream_t stream);
hipError_t launch_split(const SplitParams& p, int head_dim, int num_items, hipStream_t stream);
hipError_t launch_merge(const MergeParams& p, int head_dim, int batch, hipStream_t stream);

}  // namespace oserve
