// Shared host-side plumbing of the library: status codes, error capture and the optional
// per-kernel event timing.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/moe_circuit.h"

#include <atomic>

namespace moe {

void        note_hip_error(hipError_t e, const char* what);
bool        timing_enabled();
bool        timing_wanted(const char* kernel_name);      // timing on, and this kernel selected
void        timing_begin(const char* name, hipStream_t s);
void        timing_end(hipStream_t s);

// Brackets one kernel launch with the timing events (when enabled) and turns a launch error
// into MOE_ERR_HIP.
struct LaunchScope {
    hipStream_t s;
    bool timed;
    LaunchScope(const char* name, hipStream_t stream) : s(stream), timed(timing_wanted(name)) { if (timed) timing_begin(name, s); }
    moe_status done() {
        hipError_t e = hipGetLastError();
        if (timed) timing_end(s);
        if (e != hipSuccess) { note_hip_error(e, "kernel launch"); return MOE_ERR_HIP; }
        return MOE_OK;
    }
};

// "Done once per device" for set-up that HIP keeps per device (function attributes): bit d = done on device d.
struct DeviceOnce {
    std::atomic<unsigned long long> done{0};
    bool needed(int& dev) {
        if (hipGetDevice(&dev) != hipSuccess) dev = 0;
        return dev < 0 || dev >= 64 || !((done.load(std::memory_order_acquire) >> dev) & 1ULL);
    }
    void mark(int dev) { if (dev >= 0 && dev < 64) done.fetch_or(1ULL << dev, std::memory_order_release); }
};

}  // namespace moe

#define MOE_WAVE 64
