// Internal: how the .hip files launch a kernel that takes one by-value parameter block.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace oserve {

// Launches `kernel` on `stream` and returns the status of this launch itself.  (The launch macros
// return nothing, and asking hipGetLastError() afterwards also reports an error that an unrelated
// earlier runtime call of the thread left behind, e.g. one refused while a stream was capturing.)
// `start` / `stop`, if non-null, are attached to the kernel's dispatch: no marker packets.
template <class Params>
inline hipError_t launch_kernel(void (*kernel)(Params), dim3 grid, dim3 block, hipStream_t stream,
                                hipEvent_t start, hipEvent_t stop, const Params& p) {
    Params by_value = p;
    void* args[] = {&by_value};
    return hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, args, 0, stream, start, stop, 0);
}

}  // namespace oserve
