// Internal: the decode step's launch sequence (api.cpp), shared by the entry points that differ
// only in where the workspace comes from.
#pragma once
#include <cstddef>
#include <cstdint>

#include "oserve.h"

namespace oserve {

oserve_status_t decode_launch(oserve_plan_t* plan, void* workspace, size_t workspace_bytes, const void* q,
                              const void* k_pages, const void* v_pages, const int32_t* block_table,
                              const int32_t* context_lens, float scale, float* out, void* stream);
size_t decode_workspace_bytes(const oserve_plan_t* plan);
int decode_plan_device(const oserve_plan_t* plan);   // -1: the plan has no device

}  // namespace oserve
