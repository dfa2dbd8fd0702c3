// gfx950 kernel: causal chunked-prefill attention over the paged KV cache (one workgroup per work
// item; the work itself is in prefill_body.h, shared with the mixed prefill + decode kernel).
#include "prefill_body.h"
#include "launch_util.h"

namespace oserve {
namespace {

template <int D>
__global__ __launch_bounds__(prefill_detail::kPrefillThreads)
__attribute__((amdgpu_waves_per_eu(2, 2)))   // registers budgeted for two workgroups per compute unit
void paged_prefill_kernel(const PrefillParams p) {
    __shared__ __align__(16) unsigned char lds[prefill_detail::prefill_lds_bytes<D>()];
    prefill_detail::prefill_item_body<D>(p, p.items + blockIdx.x, (prefill_detail::lds_byte*)lds,
                                                        prefill_detail::WorkgroupBarrier{}, static_cast<int>(threadIdx.x) >> 6);
}

}  // namespace

hipError_t launch_prefill(const PrefillParams& p, int head_dim, int num_items, hipStream_t stream,
                          hipEvent_t start, hipEvent_t stop) {
    if (num_items <= 0) return hipSuccess;
    const dim3 block(prefill_detail::kPrefillThreads);
    if (head_dim == 128) return launch_kernel(paged_prefill_kernel<128>, dim3(num_items), block, stream, start, stop, p);
    if (head_dim == 64) return launch_kernel(paged_prefill_kernel<64>, dim3(num_items), block, stream, start, stop, p);
    return hipErrorInvalidValue;
}

}  // namespace oserve
