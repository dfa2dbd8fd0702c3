// gfx950 kernel: KV-block migration copies (paper section 5.2, "KV cache transmission": the KV
// blocks of long requests are moved at a deployment switch in batched, layer-aligned chunks into
// buffers pre-allocated on the target).  One layer's chunk on one GPU is two copies:
//   gather : the pages that the block table names for the migrating requests, and a range of their
//            kv heads, go from the page pool into one contiguous staging chunk
//            stage[s][j] = pool[table[row_r][s - offset_r]][head_begin + j],   offset_r <= s < offset_{r+1}
//   scatter: a staging chunk goes into the pages a (target) block table names, at a head range of
//            a pool that may hold a different number of kv heads per page (the tensor-parallel
//            degree of the target deployment may differ from the source's).
// Pure data movement, HBM-bound: every byte is read once and written once with 16-byte
// non-temporal accesses; one workgroup moves the copied heads of a whole page (contiguous on both
// sides), whose page id is found once with wave-uniform loads.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>

#include "kernels.h"
#include "launch_util.h"

namespace oserve {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kMigrateThreads = 256;

template <bool GATHER>
__global__ __launch_bounds__(kMigrateThreads) void kv_migrate_kernel(const MigrateParams p) {
    const u32x4* __restrict__ pool_or_stage_src = reinterpret_cast<const u32x4*>(blockIdx.y == 0 ? p.k_src : p.v_src);
    u32x4* __restrict__ dst = reinterpret_cast<u32x4*>(blockIdx.y == 0 ? p.k_dst : p.v_dst);
    // the copied heads of one page are contiguous both in the pool and in the staging chunk
    const int page_chunks = p.num_heads * p.unit_chunks;
    for (int64_t s = blockIdx.x; s < p.num_pages; s += gridDim.x) {
        // which table entry names the page: one 16-byte wave-uniform load
        const int4 ref = reinterpret_cast<const int4*>(p.page_refs)[s];
        const int row = p.use_source_rows ? ref.x : ref.y;
        const int pid = __builtin_amdgcn_readfirstlane(p.block_table[static_cast<int64_t>(row) * p.table_stride + ref.z]);
        const int64_t pool_off = (static_cast<int64_t>(pid) * p.pool_heads + p.head_begin) * p.unit_chunks;
        const int64_t stage_off = s * page_chunks;
        const u32x4* from = pool_or_stage_src + (GATHER ? pool_off : stage_off);
        u32x4* to = dst + (GATHER ? stage_off : pool_off);
        constexpr int U = 8;   // 16-byte loads in flight per thread: a 32 KB page in one round
        int c = threadIdx.x;
        for (; c + (U - 1) * kMigrateThreads < page_chunks; c += U * kMigrateThreads) {
            u32x4 w[U];
#pragma unroll
            for (int i = 0; i < U; ++i) w[i] = __builtin_nontemporal_load(from + c + i * kMigrateThreads);
#pragma unroll
            for (int i = 0; i < U; ++i) __builtin_nontemporal_store(w[i], to + c + i * kMigrateThreads);
        }
        for (; c < page_chunks; c += kMigrateThreads) __builtin_nontemporal_store(__builtin_nontemporal_load(from + c), to + c);
    }
}

}  // namespace

hipError_t launch_kv_migrate(const MigrateParams& p, bool gather, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop) {
    if (p.num_pages <= 0) return hipSuccess;
    // one workgroup per page and pool (measured: a short-lived workgroup per 8-32 KB span copies
    // faster than resident workgroups striding over the pages); the stride loop only serves
    // chunks beyond the grid limit
    const int64_t cap = int64_t{1} << 30;
    const dim3 grid(static_cast<unsigned>(p.num_pages < cap ? p.num_pages : cap), 2);
    if (gather) return launch_kernel(kv_migrate_kernel<true>, grid, dim3(kMigrateThreads), stream, start, stop, p);
    return launch_kernel(kv_migrate_kernel<false>, grid, dim3(kMigrateThreads), stream, start, stop, p);
}

}  // namespace oserve
