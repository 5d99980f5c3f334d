// Measurement build only (libllla_measure.so, compiled with -DLLLA_MEASURE): HIP events around every kernel a call
// enqueues, on the caller's stream.  The production library compiles the stage hooks to nothing and has no
// process-wide state; this file is not part of it.
#include "llla_common.hpp"
#include "llla_measure.h"

namespace llla {
namespace {
constexpr int kMaxStages = 16;
bool g_profile = false;
hipEvent_t g_events[kMaxStages + 1];
const char *g_names[kMaxStages];
bool g_events_ready = false;
int g_nstages = 0;
bool g_open = false;
}  // namespace

void stage_begin(hipStream_t)
{
    if (!g_profile) return;
    if (!g_events_ready) {
        for (int i = 0; i <= kMaxStages; ++i) (void)hipEventCreate(&g_events[i]);
        g_events_ready = true;
    }
    g_nstages = 0;
    g_open = false;
}

void stage_mark(hipStream_t stream, const char *name)
{
    if (!g_profile || !g_events_ready || g_nstages >= kMaxStages) return;
    (void)hipEventRecord(g_events[g_nstages], stream);
    g_names[g_nstages] = name;
    ++g_nstages;
    g_open = true;
}

void stage_end(hipStream_t stream)
{
    if (!g_profile || !g_events_ready || !g_open) return;
    (void)hipEventRecord(g_events[g_nstages], stream);
    g_open = false;
}
}  // namespace llla

extern "C" {

void llla_profile_enable(int on) { llla::g_profile = on != 0; llla::g_nstages = 0; }

int llla_profile_last(float *ms, const char **names, int max)
{
    using namespace llla;
    if (!g_profile || !g_events_ready || g_nstages == 0 || g_open) return 0;
    if (hipEventSynchronize(g_events[g_nstages]) != hipSuccess) return 0;
    int k = 0;
    for (; k < g_nstages && k < max; ++k) {
        float t = 0.f;
        (void)hipEventElapsedTime(&t, g_events[k], g_events[k + 1]);
        if (ms) ms[k] = t;
        if (names) names[k] = g_names[k];
    }
    return k;
}

}  // extern "C"
