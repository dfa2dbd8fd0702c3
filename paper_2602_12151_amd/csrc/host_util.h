// Internal: host-side helpers shared by the api_*.cpp files (device selection for the duration of a
// call, the ring of HIP event pairs behind the optional kernel timing, device facts).
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace oserve {

// Makes `dev` the current device for the lifetime of the object and restores the previous one.
struct DeviceGuard {
    int prev = -1, target = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) : target(dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~DeviceGuard() {
        if (ok && prev != target) (void)hipSetDevice(prev);
    }
    DeviceGuard(const DeviceGuard&) = delete;
    DeviceGuard& operator=(const DeviceGuard&) = delete;
};

// Optional timing of one kernel per launch call: kSlots pairs of events that a launch attaches to
// its kernel's dispatch; finished pairs are folded into a running mean.
template <int kSlots>
struct KernelTimer {
    hipEvent_t begin[kSlots] = {}, end[kSlots] = {};
    bool pending[kSlots] = {};
    bool enabled = false;
    double sum_ms = 0.0;
    int64_t count = 0;

    bool create() {
        for (int i = 0; i < kSlots; ++i)
            if (hipEventCreate(&begin[i]) != hipSuccess || hipEventCreate(&end[i]) != hipSuccess) return false;
        return true;
    }
    void destroy() {
        for (int i = 0; i < kSlots; ++i) {
            if (begin[i]) (void)hipEventDestroy(begin[i]);
            if (end[i]) (void)hipEventDestroy(end[i]);
            begin[i] = end[i] = nullptr;
        }
    }
    // Folds slot `i` into the mean if a launch is recorded in it.  Blocks until that launch's kernel has ended.
    bool collect(int i) {
        if (!pending[i]) return true;
        if (hipEventSynchronize(end[i]) != hipSuccess) return false;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, begin[i], end[i]) != hipSuccess) return false;
        sum_ms += ms;
        count += 1;
        pending[i] = false;
        return true;
    }
    bool collect_all() {
        for (int i = 0; i < kSlots; ++i)
            if (!collect(i)) return false;
        return true;
    }
    bool set_enabled(bool on) {   // also resets the mean
        if (!collect_all()) return false;
        enabled = on;
        sum_ms = 0.0;
        count = 0;
        return true;
    }
    bool mean(float* mean_ms, int32_t* n) {
        if (!collect_all()) return false;
        *n = static_cast<int32_t>(count);
        *mean_ms = count ? static_cast<float>(sum_ms / count) : 0.f;
        return true;
    }
    hipEvent_t begin_of(int i) const { return enabled ? begin[i] : nullptr; }
    hipEvent_t end_of(int i) const { return enabled ? end[i] : nullptr; }
    void mark(int i) { if (enabled) pending[i] = true; }
};

// Facts of a device that size plans.  Values the runtime cannot report are derived from ones it can.
struct DeviceFacts {
    int32_t compute_units = 0;
    int32_t xcds = 0;            // accelerator dies, each with its own L2; workgroups go to them round-robin
    int32_t simds_per_cu = 0;    // wavefront slots the split kernel fills per compute unit (one per SIMD)
};

inline bool query_device_facts(int device, DeviceFacts* out) {
    int cus = 0, xcc = 0, threads_per_cu = 0, wave = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1) return false;
    if (hipDeviceGetAttribute(&xcc, hipDeviceAttributeNumberOfXccs, device) != hipSuccess || xcc < 1) xcc = 1;
    out->compute_units = cus;
    out->xcds = xcc;
    // A compute unit of this architecture family runs at most 8 wavefronts per SIMD, so the SIMD
    // count is the resident-thread limit / (wavefront size x 8).
    out->simds_per_cu = 4;
    if (hipDeviceGetAttribute(&threads_per_cu, hipDeviceAttributeMaxThreadsPerMultiProcessor, device) == hipSuccess &&
        hipDeviceGetAttribute(&wave, hipDeviceAttributeWarpSize, device) == hipSuccess && wave > 0) {
        const int simds = threads_per_cu / (wave * 8);
        if (simds >= 1 && simds <= 16) out->simds_per_cu = simds;
    }
    return true;
}

}  // namespace oserve
