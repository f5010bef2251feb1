// Error reporting and version of the C ABI.
#include "md_host.hpp"
#include "../../include/mustdrop_bench.h"

#include <string.h>

#include <vector>

namespace md {

char* error_buffer() {
    static thread_local char buf[512] = {0};
    return buf;
}

void clear_error() { error_buffer()[0] = '\0'; }

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

namespace {
struct ProfRecord { const char* name; hipEvent_t start, stop; };
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
}  // namespace

bool profiling() { return g_prof_on; }

void profile_events(const char* kernel_name, hipEvent_t* start, hipEvent_t* stop) {
    ProfRecord r{kernel_name, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess) return;
    if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return; }
    g_prof.push_back(r);
    *start = r.start;
    *stop = r.stop;
}

}  // namespace md

extern "C" int mustdrop_profile_start(void) {
    md::clear_error();
    md::g_prof.clear();
    md::g_prof_on = true;
    return MD_OK;
}

extern "C" int mustdrop_profile_stop(char* names, float* total_ms, int* calls, int cap, int* n_out) {
    md::clear_error();
    md::g_prof_on = false;
    int n = 0;
    int rc = MD_OK;
    for (auto& r : md::g_prof) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) rc = md::fail(MD_EHIP, "profile_stop: %s", hipGetErrorString(e));
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        if (e != hipSuccess || !names || !total_ms || !calls) continue;
        int slot = -1;
        for (int i = 0; i < n; ++i)
            if (strncmp(names + 64 * i, r.name, 63) == 0) { slot = i; break; }
        if (slot < 0) {
            if (n >= cap) continue;
            slot = n++;
            strncpy(names + 64 * slot, r.name, 63);
            names[64 * slot + 63] = '\0';
            total_ms[slot] = 0.f;
            calls[slot] = 0;
        }
        total_ms[slot] += ms;
        calls[slot] += 1;
    }
    md::g_prof.clear();
    if (n_out) *n_out = n;
    return rc;
}

extern "C" const char* mustdrop_last_error(void) { return md::error_buffer(); }
extern "C" int mustdrop_version(void) { return 2; }
