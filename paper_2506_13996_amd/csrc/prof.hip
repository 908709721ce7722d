// Benchmarking and testing aids of libalst (alst_debug.h).  Per-kernel timing (alst_profile_enable /
// alst_profile_read): HIP event pairs around kernel launches, recorded on the launch stream; the
// list of spans and the pool of events are process-wide and guarded by one lock.
#include <hip/hip_runtime.h>
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/alst_debug.h"
#include "common.h"

namespace alst {

struct ProfSpan { hipEvent_t a, b; int kind; };
static std::atomic<bool> g_prof_on{false};
static std::mutex g_prof_lock;                  // guards the two vectors
static std::vector<ProfSpan> g_prof_spans;
static std::vector<hipEvent_t> g_prof_pool;

static hipEvent_t prof_event() {
    {
        std::lock_guard<std::mutex> hold(g_prof_lock);
        if (!g_prof_pool.empty()) {
            hipEvent_t e = g_prof_pool.back();
            g_prof_pool.pop_back();
            return e;
        }
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

ProfScope::ProfScope(int kind_, hipStream_t stream)
    : a(nullptr), b(nullptr), kind(kind_), s(stream), on(g_prof_on.load(std::memory_order_relaxed)) {
    if (!on) return;
    a = prof_event();
    b = prof_event();
    on = a && b;
    if (on) (void)hipEventRecord(a, s);
}

ProfScope::~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(b, s);
    std::lock_guard<std::mutex> hold(g_prof_lock);
    g_prof_spans.push_back(ProfSpan{a, b, kind});
}

// Register-resident MFMA loops for alst_debug_mfma_rate: every wavefront multiplies A and B operand
// registers it made itself into 256 accumulator registers (as the block GEMMs), with no memory
// traffic at all.  FORM16 = false: v_mfma_f32_32x32x16_bf16, 4 x 4 operands, 16 accumulator tiles;
// true: v_mfma_f32_16x16x32_bf16, 8 x 8 operands, 64 tiles.  One pass of the loop body is 2^21 flop
// per wavefront either way.  data = 0: small integers, 1: uniform in [-1, 1).
__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
template <bool FORM16>
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* __restrict__ out, int iters, int data) {
    constexpr int kOps = FORM16 ? 8 : 4;
    bf16x8_t a[kOps], b[kOps];
#pragma unroll
    for (int t = 0; t < kOps; ++t)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t ha = mix32((threadIdx.x * 16 + t) * 8 + j), hb = mix32((threadIdx.x * 16 + 8 + t + 77777) * 8 + j);
            a[t][j] = (__bf16)(data == 0 ? (float)(ha & 3) : ((int)(ha & 0xffff) - 32768) / 32768.0f);
            b[t][j] = (__bf16)(data == 0 ? (float)(hb & 3) : ((int)(hb & 0xffff) - 32768) / 32768.0f);
        }
    float s = 0.f;
    if (FORM16) {
        f32x4_t acc[64];
#pragma unroll
        for (int i = 0; i < 64; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int rep = 0; rep < 2; ++rep)
#pragma unroll
                for (int i = 0; i < 64; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 7], b[i >> 3], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 64; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) s += acc[i][j];
    } else {
        f32x16_t acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int rep = 0; rep < 4; ++rep)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[(i >> 2) & 3], acc[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) s += acc[i][j];
    }
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace alst

using namespace alst;

extern "C" {

int alst_profile_enable(int on) {
    g_prof_on.store(on != 0, std::memory_order_relaxed);
    return ALST_OK;
}

int alst_profile_read(double* ms_total, int64_t* launches) {
    if (!ms_total || !launches) return ALST_ERR_NULL;
    for (int k = 0; k < PROF_KINDS; ++k) { ms_total[k] = 0.0; launches[k] = 0; }
    int rc = ALST_OK;
    std::vector<ProfSpan> spans;
    {
        std::lock_guard<std::mutex> hold(g_prof_lock);
        spans.swap(g_prof_spans);
    }
    for (const ProfSpan& sp : spans) {              // waits for the GPU: outside the lock
        float ms = 0.f;
        if (hipEventSynchronize(sp.b) != hipSuccess ||
            hipEventElapsedTime(&ms, sp.a, sp.b) != hipSuccess) rc = ALST_ERR_HIP;
        ms_total[sp.kind] += ms;
        launches[sp.kind] += 1;
    }
    std::lock_guard<std::mutex> hold(g_prof_lock);
    for (const ProfSpan& sp : spans) {
        g_prof_pool.push_back(sp.a);
        g_prof_pool.push_back(sp.b);
    }
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

// Sustained rate of the bf16 matrix instructions the block GEMMs use, on this device now: 256
// workgroups of 4 wavefronts (one per SIMD of every compute unit) run iters * 2^21 flop each out
// of registers.  data bit 0: 0 = small-integer operands, 1 = random operands in [-1, 1) (the rate
// depends on the operand bits through the power the multipliers draw); data bit 1: 0 =
// v_mfma_f32_32x32x16_bf16 (64 per pass), 1 = v_mfma_f32_16x16x32_bf16 (128 per pass).
// scratch: 256 * 256 floats of device memory, overwritten.  Synchronises the stream.
int alst_debug_mfma_rate(int data, int iters, float* scratch, double* tflops, void* stream) {
    if (!scratch || !tflops) return ALST_ERR_NULL;
    if (iters < 1 || iters > (1 << 22) || data < 0 || data > 3) return ALST_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return ALST_ERR_HIP;
    }
    auto* const kernel = (data & 2) ? mfma_rate_kernel<true> : mfma_rate_kernel<false>;
    hipLaunchKernelGGL(kernel, dim3(256), dim3(256), 0, s, scratch, iters < 64 ? iters : 64, data & 1);   // warm-up
    (void)hipEventRecord(e0, s);
    hipLaunchKernelGGL(kernel, dim3(256), dim3(256), 0, s, scratch, iters, data & 1);
    (void)hipEventRecord(e1, s);
    float ms = 0.f;
    int rc = ALST_OK;
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
        rc = ALST_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    // per launch: 256 workgroups x 4 wavefronts x iters x 2^21 flop (64 x 2 * 32 * 32 * 16 = 128 x 2 * 16 * 16 * 32)
    *tflops = rc == ALST_OK ? 256.0 * 4.0 * (double)iters * 64.0 * 32768.0 / ((double)ms * 1e9) : 0.0;
    return rc;
}

}  // extern "C"
