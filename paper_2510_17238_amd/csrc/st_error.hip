// Error text and version of the C ABI.
#include <string.h>

#include <vector>

#include "st_internal.h"

namespace st {
static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}
const char* get_error() { return g_error; }
}  // namespace st

namespace st {
namespace {
// Kernel timing is a property of the CALLING THREAD (like the error text): a thread that switches it on gets events
// around the kernels of its own calls and reads back its own measurements; other threads are not affected.
struct Region { hipEvent_t a, b; int launches; };
thread_local bool t_prof_on = false;
thread_local int t_prof_repeat = 1;
thread_local WaveTrace t_wave_trace = {nullptr, 0};
thread_local std::vector<Region> t_regions[kProfCount];
}  // namespace

bool prof_enabled() { return t_prof_on; }
int prof_repeat() { return t_prof_on ? t_prof_repeat : 1; }
WaveTrace prof_wave_trace() { return t_prof_on ? t_wave_trace : WaveTrace{nullptr, 0}; }

void prof_begin(int which, hipStream_t stream) {
    if (!t_prof_on) return;
    Region r{};
    r.launches = t_prof_repeat;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) {
        (void)hipEventDestroy(r.a);
        return;
    }
    (void)hipEventRecord(r.a, stream);
    t_regions[which].push_back(r);
}

void prof_end(int which, hipStream_t stream) {
    if (!t_prof_on) return;
    if (!t_regions[which].empty()) (void)hipEventRecord(t_regions[which].back().b, stream);
}
}  // namespace st

extern "C" void st_profile_enable(int32_t on) { st::t_prof_on = on != 0; }
extern "C" st_status st_profile_repeat(int32_t launches) {
    if (launches < 1 || launches > 64) return st::fail(ST_ERR_INVALID_ARG, "st_profile_repeat: %d launches (1 .. 64)", launches);
    st::t_prof_repeat = launches;
    return ST_OK;
}

extern "C" st_status st_profile_wave_trace(void* device_buffer, int32_t n_pairs) {
    if (device_buffer && (n_pairs <= 0 || (reinterpret_cast<uintptr_t>(device_buffer) & 15u)))
        return st::fail(ST_ERR_INVALID_ARG, "st_profile_wave_trace: buffer must be 16-byte aligned and hold at least one pair");
    st::t_wave_trace = st::WaveTrace{static_cast<unsigned long long*>(device_buffer), device_buffer ? n_pairs : 0};
    return ST_OK;
}

extern "C" st_status st_profile_read(int32_t which, double* mean_ms, int32_t* count) {
    using namespace st;
    if (which < 0 || which >= kProfCount || !mean_ms || !count) return fail(ST_ERR_INVALID_ARG, "st_profile_read: bad argument");
    double total = 0.0;
    int n = 0;
    for (Region& r : t_regions[which]) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            total += ms / r.launches;
            ++n;
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    t_regions[which].clear();
    *mean_ms = n ? total / n : 0.0;
    *count = n;
    return ST_OK;
}

extern "C" const char* st_last_error(void) { return st::get_error(); }
extern "C" int32_t st_version(void) { return 2; }
