// Optional per-kernel timing with HIP events attached to the kernel dispatches.

#include <vector>

#include "qadc_common.h"
#include "qadc_profile.h"

namespace qadc {

namespace {
struct Pair { hipEvent_t a, b; int which; };
bool g_on = false;
int g_only = -1;  // >= 0: only this slot is timed
std::vector<Pair> g_open;
std::vector<hipEvent_t> g_free;   // events kept for reuse: creating one costs host time per launch
double g_ms[QADC_PROF_COUNT];
int64_t g_launches[QADC_PROF_COUNT];
}  // namespace

bool prof_open(int which, hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_on || (g_only >= 0 && which != g_only)) return false;
    Pair p;
    p.which = which;
    hipEvent_t *ev[2] = {&p.a, &p.b};
    for (int i = 0; i < 2; ++i) {
        if (!g_free.empty()) {
            *ev[i] = g_free.back();
            g_free.pop_back();
        } else if (hipEventCreate(ev[i]) != hipSuccess) {
            if (i) g_free.push_back(p.a);
            return false;
        }
    }
    g_open.push_back(p);
    *start = p.a;
    *stop = p.b;
    return true;
}

static void drain()
{
    for (Pair &p : g_open) {
        float ms = 0.f;
        if (hipEventSynchronize(p.b) == hipSuccess && hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
            g_ms[p.which] += ms;
            g_launches[p.which] += 1;
        }
        g_free.push_back(p.a);
        g_free.push_back(p.b);
    }
    g_open.clear();
}

int profile_enable(int on)
{
    drain();
    if (on) {
        for (int i = 0; i < QADC_PROF_COUNT; ++i) { g_ms[i] = 0; g_launches[i] = 0; }
    }
    g_on = on != 0;
    g_only = -1;
    return QADC_OK;
}

int profile_only(int which)
{
    if (which < 0 || which >= QADC_PROF_COUNT) return fail(QADC_EINVAL, "qadc_profile_only: bad slot %d", which);
    const int rc = profile_enable(1);
    g_only = which;
    return rc;
}

int profile_read(int which, double *total_ms, int64_t *launches)
{
    if (which < 0 || which >= QADC_PROF_COUNT || !total_ms || !launches)
        return fail(QADC_EINVAL, "qadc_profile_read: bad argument");
    drain();
    *total_ms = g_ms[which];
    *launches = g_launches[which];
    return QADC_OK;
}

}  // namespace qadc
