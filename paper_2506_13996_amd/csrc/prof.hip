// Per-kernel timing aid of libalst (alst_profile_enable / alst_profile_read): HIP event pairs around
// kernel launches, recorded on the launch stream.  Process-wide state, not thread-safe.
#include <hip/hip_runtime.h>
#include <vector>

#include "common.h"

namespace alst {

struct ProfSpan { hipEvent_t a, b; int kind; };
static bool g_prof_on = false;
static std::vector<ProfSpan> g_prof_spans;
static std::vector<hipEvent_t> g_prof_pool;

static hipEvent_t prof_event() {
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

ProfScope::ProfScope(int kind_, hipStream_t stream) : a(nullptr), b(nullptr), kind(kind_), s(stream), on(g_prof_on) {
    if (!on) return;
    a = prof_event();
    b = prof_event();
    on = a && b;
    if (on) (void)hipEventRecord(a, s);
}

ProfScope::~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(b, s);
    g_prof_spans.push_back(ProfSpan{a, b, kind});
}

}  // namespace alst

using namespace alst;

extern "C" {

int alst_profile_enable(int on) {
    g_prof_on = on != 0;
    return ALST_OK;
}

int alst_profile_read(double* ms_total, int64_t* launches) {
    if (!ms_total || !launches) return ALST_ERR_NULL;
    for (int k = 0; k < PROF_KINDS; ++k) { ms_total[k] = 0.0; launches[k] = 0; }
    int rc = ALST_OK;
    for (const ProfSpan& sp : g_prof_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(sp.b) != hipSuccess ||
            hipEventElapsedTime(&ms, sp.a, sp.b) != hipSuccess) rc = ALST_ERR_HIP;
        ms_total[sp.kind] += ms;
        launches[sp.kind] += 1;
        g_prof_pool.push_back(sp.a);
        g_prof_pool.push_back(sp.b);
    }
    g_prof_spans.clear();
    return rc;
}

}  // extern "C"
