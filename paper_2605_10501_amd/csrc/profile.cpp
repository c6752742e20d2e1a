// Optional per-launch timing: HIP events around each kernel launch on the launch stream (ms_profile_*).
// Process-wide state without locking: enable, launch and read from one thread at a time.
#include <vector>

#include "common.h"
#include "launch.h"

// ---- per-launch timing ----------------------------------------------------------------------
namespace {
constexpr int kMaxProf = 16384;
struct ProfRec { hipEvent_t a, b; int cls; double work; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
}  // namespace

void prof_begin(int cls, double work, hipStream_t s, int *slot) {
    *slot = -1;
    if (!g_prof_on || (int)g_prof.size() >= kMaxProf) return;
    ProfRec r;
    r.cls = cls;
    r.work = work;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    (void)hipEventRecord(r.a, s);
    g_prof.push_back(r);
    *slot = (int)g_prof.size() - 1;
}

void prof_end(int slot, hipStream_t s) { (void)hipEventRecord(g_prof[slot].b, s); }

extern "C" ms_status ms_profile_enable(int32_t on) {
    for (auto &r : g_prof) {
        (void)hipEventSynchronize(r.b);
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
    g_prof_on = on != 0;
    return MS_OK;
}

extern "C" ms_status ms_profile_read(int32_t cls, int64_t *launches, double *total_ms, double *total_work) {
    if (!launches || !total_ms || !total_work || cls < 0 || cls >= MS_PROFILE_CLASSES)
        return ms_fail(MS_ERR_INVALID_ARG, "profile_read: bad argument");
    *launches = 0;
    *total_ms = 0.0;
    *total_work = 0.0;
    for (auto &r : g_prof) {
        if (r.cls != cls) continue;
        MS_CHECK_HIP(hipEventSynchronize(r.b));
        float ms = 0.f;
        MS_CHECK_HIP(hipEventElapsedTime(&ms, r.a, r.b));
        *launches += 1;
        *total_ms += ms;
        *total_work += r.work;
    }
    return MS_OK;
}
