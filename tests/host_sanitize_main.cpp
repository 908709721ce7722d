// Host-side logic of libalst under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).
//
// Built by tests/test_abi_host.py from the library's own sources with the sanitizers on the host
// pass; no kernel is ever launched: every call below either is pure host arithmetic (workspace
// sizing, the workgroup -> output block mapping) or is stopped by the argument validation before
// anything is enqueued (the pointers are fakes, the workspace is one byte too small).  What runs
// under the sanitizers is therefore the layout arithmetic, the choice of dHidden ranges for every
// row count, the patch-shape choice and the grid-size checks, over a sweep of shapes that
// includes ragged, tiny and maximal extents.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "alst.h"
#include "alst_debug.h"
#include "alst_linear.h"
#include "alst_mlp.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            ++failures;                                                     \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond);      \
        }                                                                   \
    } while (0)

static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }

int main() {
    const int64_t Ns[] = {1, 5, 255, 256, 257, 1000, 4096, 32768, 131072, 524288, (int64_t)1 << 30};
    const int64_t Hs[] = {8, 64, 136, 256, 1600, 2880, 4096, 5120, 8192, (int64_t)1 << 20};
    const int64_t Vs[] = {1, 2, 7, 72, 255, 256, 1000, 4096, 50257, 128256, 151936, 152064, (int64_t)1 << 24};
    const int64_t Ts[] = {1, 77, 128, 256, 300, 2048, 4096, 8192, 16384, 65536, (int64_t)1 << 30};
    const uint32_t Fs[] = {0u, ALST_FLAG_DW_FP32, ALST_FLAG_DW_FP32 | ALST_FLAG_DW_ACCUMULATE,
                           ALST_FLAG_TILE_SCRATCH, ALST_FLAG_TILE_SCRATCH | ALST_FLAG_REDUCE_SUM,
                           ALST_FLAG_FORWARD_ONLY};
    long calls = 0;
    for (int64_t N : Ns)
        for (int64_t H : Hs)
            for (int64_t V : Vs)
                for (int64_t T : Ts)
                    for (uint32_t f : Fs) {
                        const size_t w = alst_tiled_ce_workspace_bytes(N, H, V, T, f);
                        EXPECT(w > 0);
                        ++calls;
                        // one byte short: the validation runs through every shape check and
                        // returns before anything is launched (ALST_ERR_SHAPE where a launch
                        // would not fit a grid)
                        const int rc = alst_tiled_ce_forward(fake(0x10000), fake(0x20000),
                                                             static_cast<const int32_t*>(fake(0x30000)), N, H, V,
                                                             T, -100, static_cast<float*>(fake(0x40000)),
                                                             nullptr, nullptr, fake(0x50000), w - 1, f,
                                                             nullptr);
                        EXPECT(rc == ALST_ERR_WORKSPACE || rc == ALST_ERR_SHAPE);
                        if (!(f & ALST_FLAG_FORWARD_ONLY)) {
                            const int rb = alst_tiled_ce_forward_backward(
                                fake(0x10000), fake(0x20000), static_cast<const int32_t*>(fake(0x30000)), N, H,
                                V, T, -100, 1.f, static_cast<float*>(fake(0x40000)), nullptr, nullptr,
                                fake(0x60000), fake(0x70000), fake(0x50000), w - 1, f, nullptr);
                            EXPECT(rb == rc);
                        }
                        const int rt = alst_tiled_ce_token_losses(fake(0x50000), w - 1, N, H, V, T, f,
                                                                  static_cast<float*>(fake(0x80000)), nullptr);
                        EXPECT(rt == ALST_ERR_WORKSPACE);
                    }
    // invalid shapes and flags size to 0
    EXPECT(alst_tiled_ce_workspace_bytes(0, 64, 64, 64, 0) == 0);
    EXPECT(alst_tiled_ce_workspace_bytes(((int64_t)1 << 30) + 1, 64, 64, 64, 0) == 0);
    EXPECT(alst_tiled_ce_workspace_bytes(64, 64, ((int64_t)1 << 24) + 1, 64, 0) == 0);
    EXPECT(alst_tiled_ce_workspace_bytes(64, 64, 64, 64, 1u << 20) == 0);

    // tiled MLP and tiled linear layer: sizing and validation
    const int64_t Is[] = {8, 96, 128, 1000, 14336, 27648};
    for (int64_t N : {(int64_t)1, (int64_t)300, (int64_t)256000, (int64_t)1 << 22})
        for (int64_t H : {(int64_t)8, (int64_t)136, (int64_t)4096, (int64_t)5120})
            for (int64_t I : Is)
                for (int64_t T : {(int64_t)1, (int64_t)300, (int64_t)4096, (int64_t)1 << 22})
                    for (uint32_t f : {0u, (uint32_t)ALST_FLAG_DW_FP32}) {
                        const size_t wf = alst_tiled_mlp_workspace_bytes(N, H, I, T, 0, f);
                        const size_t wb = alst_tiled_mlp_workspace_bytes(N, H, I, T, 1, f);
                        EXPECT(wf > 0 && wb > wf);
                        calls += 2;
                        EXPECT(alst_tiled_mlp_forward(fake(0x10000), fake(0x20000), fake(0x30000),
                                                      fake(0x40000), N, H, I, T, fake(0x50000), fake(0x60000),
                                                      wf - 1, f, nullptr) == ALST_ERR_WORKSPACE);
                        EXPECT(alst_tiled_mlp_backward(fake(0x10000), fake(0x20000), fake(0x30000),
                                                       fake(0x40000), fake(0x50000), N, H, I, T, fake(0x60000),
                                                       fake(0x70000), fake(0x80000), fake(0x90000),
                                                       fake(0xa0000), wb - 1, f, nullptr) == ALST_ERR_WORKSPACE);
                        const size_t wl = alst_tiled_linear_workspace_bytes(N, H, I, T, 1, f);
                        EXPECT((wl == 0) == (f == ALST_FLAG_DW_FP32 && I % 64 != 0));     // sums in dW, W as it is
                        if (wl)
                            EXPECT(alst_tiled_linear_backward(fake(0x10000), fake(0x20000), fake(0x30000), N,
                                                              H, I, T, fake(0x40000), fake(0x50000),
                                                              fake(0x60000), wl - 1, f,
                                                              nullptr) == ALST_ERR_WORKSPACE);
                    }

    // workgroup -> output block mapping: every block of every part exactly once
    const int shapes[][3] = {{16, 501, 1}, {16, 16, 1}, {8, 16, 2}, {20, 594, 1}, {16, 56, 3},
                             {3, 5, 4},    {1, 1, 8},   {17, 3, 5}, {1, 40, 1},   {64, 2, 1}};
    for (const auto& sh : shapes) {
        const int tr_n = sh[0], tc_n = sh[1], parts = sh[2];
        int part, tr, tc;
        const int n = alst_debug_block_tile(tr_n, tc_n, parts, 0, &part, &tr, &tc);
        EXPECT(n > 0 && n % 256 == 0);
        unsigned char* seen = static_cast<unsigned char*>(calloc((size_t)tr_n * tc_n * parts, 1));
        long covered = 0;
        for (int bid = 0; bid < n; ++bid) {
            EXPECT(alst_debug_block_tile(tr_n, tc_n, parts, bid, &part, &tr, &tc) == n);
            if (part < 0) continue;
            EXPECT(part < parts && tr >= 0 && tr < tr_n && tc >= 0 && tc < tc_n);
            unsigned char& s = seen[((size_t)part * tr_n + tr) * tc_n + tc];   // out of range: ASan reports
            EXPECT(s == 0);
            s = 1;
            ++covered;
        }
        EXPECT(covered == (long)tr_n * tc_n * parts);
        free(seen);
    }
    printf("host_sanitize: %ld sizing calls, %d failures\n", calls, failures);
    return failures ? 1 : 0;
}
