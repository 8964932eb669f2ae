// Per-launch HIP-event timing (see profile.h) and its two C entry points.
#include "profile.h"
#include <vector>
#include "../../include/fise.h"

namespace fise {
int fail(int code, const char* fmt, ...);

bool g_profile_on = false;
namespace {
struct Rec { int kind; double flops, bytes; hipEvent_t a, b; };
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
hipEvent_t take_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

void profile_begin(int kind, double flops, double bytes, hipStream_t st) {
    Rec r{kind, flops, bytes, take_event(), take_event()};
    if (r.a) (void)hipEventRecord(r.a, st);
    g_recs.push_back(r);
}
void profile_end(hipStream_t st) {
    if (g_recs.empty()) return;
    Rec& r = g_recs.back();
    if (r.b) (void)hipEventRecord(r.b, st);
}
}  // namespace fise

using namespace fise;

extern "C" int fise_profile_enable(int on) {
    g_profile_on = on != 0;
    return FISE_OK;
}

extern "C" int fise_profile_calibrate(int n, void* stream) {
    if (n < 0) return fail(FISE_ERR_SHAPE, "fise_profile_calibrate: n=%d", n);
    const bool was = g_profile_on;
    g_profile_on = true;
    for (int i = 0; i < n; ++i) { ProfileScope empty(PROF_EMPTY, 0.0, 0.0, (hipStream_t)stream); }
    g_profile_on = was;
    return FISE_OK;
}

extern "C" int fise_profile_read(int kind, double* total_ms, double* total_flops, double* total_bytes, int* launches) {
    if (!total_ms || !total_flops || !total_bytes || !launches) return fail(FISE_ERR_NULL, "fise_profile_read: null pointer");
    if (kind < -1 || kind >= PROF_KINDS) return fail(FISE_ERR_SHAPE, "fise_profile_read: kind %d", kind);
    *total_ms = 0; *total_flops = 0; *total_bytes = 0; *launches = 0;
    if (kind == -1) {                                   // reset: wait for and recycle every event
        for (Rec& r : g_recs) {
            if (r.b) (void)hipEventSynchronize(r.b);
            if (r.a) g_pool.push_back(r.a);
            if (r.b) g_pool.push_back(r.b);
        }
        g_recs.clear();
        return FISE_OK;
    }
    for (Rec& r : g_recs) {
        if (r.kind != kind || !r.a || !r.b) continue;
        if (hipEventSynchronize(r.b) != hipSuccess) return fail(FISE_ERR_HIP, "fise_profile_read: event synchronize failed");
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return fail(FISE_ERR_HIP, "fise_profile_read: elapsed time failed");
        *total_ms += ms; *total_flops += r.flops; *total_bytes += r.bytes; *launches += 1;
    }
    return FISE_OK;
}
