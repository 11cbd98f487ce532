// Optional per-stage kernel timing: while a profile is open every kernel launch of the library is
// issued with a start/stop event pair that the runtime stamps with the dispatch's own begin and end
// times, so the sums exclude launch gaps.  Off by default; the normal path pays one branch per launch.
#include "poly_dev.h"

#include <vector>

namespace {
struct Record { int stage; hipEvent_t a, b; };
std::vector<Record> g_pool;
size_t g_used = 0;
bool g_on = false;
}  // namespace

bool poly_prof_next(int stage, hipEvent_t *a, hipEvent_t *b)
{
    if (!g_on || g_used >= g_pool.size()) return false;
    Record &r = g_pool[g_used++];
    r.stage = stage;
    *a = r.a;
    *b = r.b;
    return true;
}

extern "C" int poly_profile_begin(int max_launches)
{
    if (g_on || max_launches <= 0 || max_launches > (1 << 20)) return POLY_EINVAL;
    g_pool.resize((size_t)max_launches);
    for (size_t i = 0; i < g_pool.size(); ++i) {
        if (hipEventCreate(&g_pool[i].a) != hipSuccess || hipEventCreate(&g_pool[i].b) != hipSuccess) {
            g_pool.resize(i);
            break;
        }
    }
    g_used = 0;
    g_on = true;
    return POLY_OK;
}

extern "C" int poly_profile_end(poly_profile *out)
{
    if (!g_on || !out) return POLY_EINVAL;
    g_on = false;
    int rc = hipDeviceSynchronize() == hipSuccess ? POLY_OK : POLY_EHIP;
    for (int s = 0; s < POLY_STAGE_COUNT; ++s) { out->launches[s] = 0; out->ms[s] = 0.f; }
    out->dropped = 0;
    for (size_t i = 0; i < g_used && rc == POLY_OK; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_pool[i].a, g_pool[i].b) != hipSuccess) { out->dropped++; continue; }
        out->launches[g_pool[i].stage]++;
        out->ms[g_pool[i].stage] += ms;
    }
    for (Record &r : g_pool) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_pool.clear();
    g_used = 0;
    return rc;
}
