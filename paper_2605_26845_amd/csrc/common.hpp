// Shared host-side plumbing of the library: status codes, error capture and the optional
// per-kernel event timing.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/moe_circuit.h"

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

}  // namespace moe

#define MOE_WAVE 64
