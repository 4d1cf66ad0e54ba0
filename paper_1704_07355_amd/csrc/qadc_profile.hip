// Optional per-kernel timing with HIP events attached to the kernel dispatches.

#include <vector>

#include "qadc_common.h"
#include "qadc_profile.h"

namespace qadc {

namespace {
struct Pair { hipEvent_t a, b; int which; };
bool g_on = false;
std::vector<Pair> g_open;
double g_ms[QADC_PROF_COUNT];
int64_t g_launches[QADC_PROF_COUNT];
}  // namespace

bool prof_open(int which, hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_on) return false;
    Pair p;
    p.which = which;
    if (hipEventCreate(&p.a) != hipSuccess) return false;
    if (hipEventCreate(&p.b) != hipSuccess) { (void)hipEventDestroy(p.a); return false; }
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
        (void)hipEventDestroy(p.a);
        (void)hipEventDestroy(p.b);
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
    return QADC_OK;
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
