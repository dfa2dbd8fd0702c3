// The decode step for callers that cannot allocate device memory (code that runs while a HIP graph
// capture is in progress, tight serving loops, harnesses that forbid hipMalloc): the same launch sequence as
// oserve_paged_decode_attn, with the workspace taken from a fixed array in device memory instead
// of from the caller.
//
// The array below lives in every GPU's memory from the moment the library's code object is loaded
// on it until the process ends.  In host code its name is only a handle for the runtime, not a
// device address: the address is asked for once per device (with that device current) and kept,
// and host code uses nothing but that address afterwards.
#include <hip/hip_runtime.h>

#include <mutex>

#include "decode_launch.h"
#include "host_util.h"
#include "oserve.h"

namespace {

static __device__ __align__(256) unsigned char scratch[OSERVE_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: the address of its copy of `scratch`

// The address of `device`'s copy of the array; resolved on the first call for that device.
oserve_status_t scratch_of(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return OSERVE_ERR_PLAN_MISMATCH;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[device]) {
        oserve::DeviceGuard guard(device);
        if (!guard.ok) return OSERVE_ERR_DEVICE;
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return OSERVE_ERR_DEVICE;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return OSERVE_OK;
}

}  // namespace

extern "C" {

size_t oserve_static_workspace_bytes(void) { return OSERVE_STATIC_WORKSPACE_BYTES; }

oserve_status_t oserve_static_workspace_init(int32_t device_id) {
    void* p = nullptr;
    return scratch_of(device_id, &p);
}

oserve_status_t oserve_paged_decode_attn_static(oserve_plan_t* plan, const void* q, const void* k_pages,
                                                const void* v_pages, const int32_t* block_table,
                                                const int32_t* context_lens, float scale, float* out,
                                                void* stream) {
    if (!plan) return OSERVE_ERR_NULL;
    if (oserve::decode_workspace_bytes(plan) > OSERVE_STATIC_WORKSPACE_BYTES) return OSERVE_ERR_WORKSPACE;
    void* ws = nullptr;
    const oserve_status_t st = scratch_of(oserve::decode_plan_device(plan), &ws);
    if (st != OSERVE_OK) return st;
    // Nothing in the workspace has to start at zero: the expand kernel writes every descriptor and
    // request record the later kernels read, and the split kernel writes every partial row the
    // merge kernel reads, so whatever the previous call left behind is never looked at.
    return oserve::decode_launch(plan, ws, OSERVE_STATIC_WORKSPACE_BYTES, q, k_pages, v_pages, block_table,
                                 context_lens, scale, out, stream);
}

}  // extern "C"
