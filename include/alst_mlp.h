/*
 * alst_mlp.h -- C ABI of the MI355X (gfx950) sequence-tiled MLP block.
 *
 * The operation (ALST paper, subsection "TiledMLP" of "Sequence Tiling for Reducing Activation
 * Memory Footprint"): the MLP of a transformer layer has no cross-sequence dependency, so its
 * forward and backward are run tile by tile along the sequence and the [tile, intermediate]
 * activations exist only for the tile in flight; backward recomputes them from the tile's input.
 * The result equals the untiled MLP.  The MLP is the gated one of the paper's example (the
 * Llama-8B MLP layer on a [256 000, 4096] bf16 input, tile = hidden size):
 *
 *   g = x Wg^T,  u = x Wu^T          x [N,H],  Wg, Wu [I,H]
 *   a = silu(g) * u                  silu(z) = z / (1 + exp(-z))
 *   y = a Wd^T                       Wd [H,I],  y [N,H]
 *
 *   da = dy Wd,  dg = da * u * silu'(g),  du = da * silu(g)
 *   dx = dg Wg + du Wu,  dWg = dg^T x,  dWu = du^T x,  dWd = dy^T a
 *
 * Products are bf16 x bf16 with fp32 accumulation; g and u enter the SwiGLU as fp32 accumulators
 * and never reach memory; a, da, dg, du are rounded to bf16 between the contractions (as a bf16
 * framework would); weight gradients are accumulated over the tiles in fp32.
 *
 * Conventions are those of alst.h: device pointers unless marked host, dense row-major without
 * strides, bf16 = upper half of an IEEE binary32, H and I multiples of 8 and base pointers 16-byte
 * aligned (else ALST_ERR_ALIGN), the caller owns every buffer including `workspace`, calls
 * validate on the host, enqueue on `stream` (a hipStream_t passed as void*) and return without
 * synchronising, and return an alst_status.  tile: any value >= 1, clamped to N; N need not be a
 * multiple of it; it changes memory and scheduling only.
 */
#ifndef ALST_MLP_H
#define ALST_MLP_H

#include "alst.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Bytes of device scratch alst_tiled_mlp_forward (backward = 0) or alst_tiled_mlp_backward
 * (backward = 1) needs, 0 if the shape is invalid.  Pure host arithmetic.  Independent of N:
 * O(tile * I) for the activations of the tiles in flight, plus O(H * I) in backward: the fp32
 * weight-gradient sums (12 H I bytes; absent for fp32 overwrite outputs) and, for H and I that
 * are multiples of 64, bf16 copies of the three weight matrices transposed (6 H I bytes, made once
 * per call, so that the products with a weight over its row index read it along its rows).
 */
size_t alst_tiled_mlp_workspace_bytes(int64_t N, int64_t H, int64_t I, int64_t tile, int backward,
                                      uint32_t flags);

/*
 * y = (silu(x Wg^T) * (x Wu^T)) Wd^T, tile by tile (6 N H I flop).
 *   x [N,H], Wg [I,H], Wu [I,H], Wd [H,I] bf16     inputs, not modified
 *   y [N,H] bf16                                   overwritten
 */
int alst_tiled_mlp_forward(const void* x, const void* Wg, const void* Wu, const void* Wd,
                           int64_t N, int64_t H, int64_t I, int64_t tile, void* y,
                           void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Gradients for upstream dy [N,H] bf16; each tile's g and u are recomputed (16 N H I flop).
 *   dx [N,H] bf16                        overwritten
 *   dWg, dWu [I,H], dWd [H,I]            bf16 (fp32 with ALST_FLAG_DW_FP32); overwritten, or += with
 *                                        ALST_FLAG_DW_ACCUMULATE
 */
int alst_tiled_mlp_backward(const void* x, const void* Wg, const void* Wu, const void* Wd,
                            const void* dy, int64_t N, int64_t H, int64_t I, int64_t tile,
                            void* dx, void* dWg, void* dWu, void* dWd,
                            void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ALST_MLP_H */
