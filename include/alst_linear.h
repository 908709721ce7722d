/*
 * alst_linear.h -- C ABI of the MI355X (gfx950) sequence-tiled linear layer.
 *
 * The operation (ALST paper, section "Sequence Tiling for Reducing Activation Memory Footprint":
 * linear layers are among the operations without cross-sequence dependency that can be run on
 * tiles of the sequence; the generic form of the paper's tiled computation applied to one
 * projection):
 *
 *   y = x W^T                 x [N,K], W [M,K], y [N,M]
 *   dx = dy W,  dW = dy^T x   dy [N,M]
 *
 * bf16 operands, fp32 accumulation; dW is accumulated over the tiles in fp32.  Conventions are
 * those of alst.h (device pointers, dense row-major, K and M multiples of 8, 16-byte aligned base
 * pointers, caller-owned workspace, asynchronous on `stream`, alst_status return values).  x and
 * dy are read as they are by every product (no activation is copied or transposed), so the forward
 * pass needs no workspace; the backward pass needs the fp32 dW sums (4 M K bytes; none with fp32
 * overwrite output, whose sums live in dW) and, for M a multiple of 64, a bf16 copy of W transposed
 * (2 M K bytes, made once per call).  `workspace` may be NULL when none is needed.
 */
#ifndef ALST_LINEAR_H
#define ALST_LINEAR_H

#include "alst.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of device scratch for forward (backward = 0: always 0) or backward (backward = 1);
 * independent of N and of the tile: 4 M K for the fp32 dW sums (absent for fp32 overwrite output,
 * whose sums live in dW) and, for M a multiple of 64, 2 M K for a bf16 copy of W transposed (made
 * once per call, so that dx = dy W reads both operands along their rows).  Pure host arithmetic;
 * 0 also for an invalid shape. */
size_t alst_tiled_linear_workspace_bytes(int64_t N, int64_t K, int64_t M, int64_t tile, int backward,
                                         uint32_t flags);

/* y [N,M] bf16 = x W^T, tile by tile (2 N K M flop). */
int alst_tiled_linear_forward(const void* x, const void* W, int64_t N, int64_t K, int64_t M,
                              int64_t tile, void* y, void* workspace, size_t workspace_bytes,
                              uint32_t flags, void* stream);

/* dx [N,K] bf16 = dy W (overwritten); dW [M,K] = dy^T x, bf16 (fp32 with ALST_FLAG_DW_FP32),
 * overwritten or += with ALST_FLAG_DW_ACCUMULATE (4 N K M flop). */
int alst_tiled_linear_backward(const void* x, const void* W, const void* dy, int64_t N, int64_t K,
                               int64_t M, int64_t tile, void* dx, void* dW, void* workspace,
                               size_t workspace_bytes, uint32_t flags, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ALST_LINEAR_H */
