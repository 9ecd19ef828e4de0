// Error text capture and the optional per-kernel event timing table.
#include "common.hpp"
#include <string.h>
#include <stdio.h>
#include <vector>

namespace moe {

static char g_err[256] = "";
static bool g_timing = false;
static char g_only[64] = "";      // when not empty: the one kernel whose launches are timed

struct Span { const char* name; hipEvent_t a, b; };
static std::vector<Span> g_spans;
static std::vector<hipEvent_t> g_pool;
static Span g_open = {nullptr, nullptr, nullptr};

void note_hip_error(hipError_t e, const char* what) {
    snprintf(g_err, sizeof(g_err), "%s: %s", what, hipGetErrorString(e));
}
bool timing_enabled() { return g_timing; }
bool timing_wanted(const char* kernel_name) { return g_timing && (g_only[0] == 0 || strcmp(g_only, kernel_name) == 0); }

static hipEvent_t get_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    // timing only: nothing synchronises with these events, so they need no system-scope fence (which would add a
    // cache write-back and invalidation to the stream at both ends of every timed kernel)
    hipError_t rc = hipEventCreateWithFlags(&e, hipEventDisableSystemFence);
    if (rc != hipSuccess) { note_hip_error(rc, "hipEventCreateWithFlags"); return nullptr; }
    return e;
}

void timing_begin(const char* name, hipStream_t s) {
    g_open.name = name; g_open.a = get_event(); g_open.b = get_event();
    if (g_open.a) (void)hipEventRecord(g_open.a, s);
}
void timing_end(hipStream_t s) {
    if (g_open.b) (void)hipEventRecord(g_open.b, s);
    if (g_open.a && g_open.b) g_spans.push_back(g_open);
    g_open = {nullptr, nullptr, nullptr};
}

}  // namespace moe

extern "C" moe_status moe_kernel_timing_enable(int on) {
    moe::g_timing = on != 0;
    return MOE_OK;
}

extern "C" moe_status moe_kernel_timing_select(const char* kernel_name) {
    if (kernel_name && strlen(kernel_name) >= sizeof(moe::g_only)) return MOE_ERR_INVALID_ARG;
    if (kernel_name) strcpy(moe::g_only, kernel_name); else moe::g_only[0] = 0;
    return MOE_OK;
}

extern "C" int moe_kernel_timing_read(const char** names, float* total_ms, int* launches, int cap) {
    if (cap < 0 || (cap > 0 && (!names || !total_ms || !launches))) return MOE_ERR_INVALID_ARG;
    int n = 0;
    moe_status st = MOE_OK;
    for (auto& sp : moe::g_spans) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(sp.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, sp.a, sp.b);
        if (e != hipSuccess) { moe::note_hip_error(e, "event timing"); st = MOE_ERR_HIP; }
        int k = 0;
        while (k < n && strcmp(names[k], sp.name) != 0) ++k;
        if (k == n) {
            if (n == cap) { moe::g_pool.push_back(sp.a); moe::g_pool.push_back(sp.b); continue; }
            names[n] = sp.name; total_ms[n] = 0.f; launches[n] = 0; ++n;
        }
        total_ms[k] += ms; launches[k] += 1;
        moe::g_pool.push_back(sp.a); moe::g_pool.push_back(sp.b);
    }
    moe::g_spans.clear();
    return st == MOE_OK ? n : st;
}

extern "C" const char* moe_last_hip_error(void) { return moe::g_err; }
