#include "prof.hpp"

#include <vector>

#include "../../include/tpi.h"
#include "host_util.hpp"

namespace tpi {

static int g_stage = kStageNone;
static std::vector<hipEvent_t> g_start, g_stop;
static size_t g_used = 0;
static bool g_open = false;

void prof_begin(int stage, hipStream_t st)
{
    if (stage != g_stage || g_used >= g_start.size()) return;
    if (hipEventRecord(g_start[g_used], st) == hipSuccess) g_open = true;
}

void prof_end(int stage, hipStream_t st)
{
    if (stage != g_stage || !g_open) return;
    g_open = false;
    if (hipEventRecord(g_stop[g_used], st) == hipSuccess) ++g_used;
}

}  // namespace tpi

using namespace tpi;

extern "C" {

int tpi_prof_enable(int stage, int32_t capacity)
{
    if (stage < 0 || stage >= kStageCount) return fail(TPI_EINVAL, "unknown stage %d", stage);
    if (capacity < 0 || capacity > (1 << 20)) return fail(TPI_EINVAL, "capacity %d out of range", capacity);
    g_stage = kStageNone;
    g_used = 0;
    g_open = false;
    if (stage == kStageNone) return TPI_OK;
    while ((int32_t)g_start.size() < capacity) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return fail(TPI_ERUNTIME, "hipEventCreate failed");
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(TPI_ERUNTIME, "hipEventCreate failed"); }
        g_start.push_back(a);
        g_stop.push_back(b);
    }
    g_stage = stage;
    return TPI_OK;
}

int tpi_prof_read(double *total_ms, int32_t *launches)
{
    double tot = 0.0;
    for (size_t i = 0; i < g_used; ++i) {
        hipError_t e = hipEventSynchronize(g_stop[i]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_start[i], g_stop[i]);
        if (e != hipSuccess) return fail(TPI_ERUNTIME, "event %zu: %s", i, hipGetErrorString(e));
        tot += ms;
    }
    if (total_ms) *total_ms = tot;
    if (launches) *launches = (int32_t)g_used;
    g_used = 0;
    return TPI_OK;
}

}  // extern "C"

