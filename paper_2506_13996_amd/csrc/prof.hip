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

// The workgroup -> output block mapping of the block GEMM launches, evaluated on the host with the
// functions the kernels use (gemm_tile.h), for a launch of `parts` products of tiles_r x tiles_c
// blocks each.  Returns the launch's number of workgroups (< 0: alst_status); for workgroup `bid`
// writes the part and the block it works on, part = -1 for a workgroup that leaves at once.
int alst_debug_block_tile(int tiles_r, int tiles_c, int parts, int bid, int* part, int* tr, int* tc) {
    if (!part || !tr || !tc) return -ALST_ERR_NULL;
    if (tiles_r < 1 || tiles_c < 1 || parts < 1 || bid < 0) return -ALST_ERR_SHAPE;
    const PatchGrid g = choose_patches(tiles_r, tiles_c);
    const int64_t total = (int64_t)g.patches() * parts;
    if (total * 32 > 0x7fffff00) return -ALST_ERR_SHAPE;
    int P, w;
    patch_of_block(bid, P, w);
    *part = -1; *tr = 0; *tc = 0;
    if (P < total) {
        const int which = P / g.patches();
        int r, c;
        if (tile_in_patch(g, P - which * g.patches(), w, r, c)) { *part = which; *tr = r; *tc = c; }
    }
    return grid_for_patches(total);
}

}  // extern "C"
