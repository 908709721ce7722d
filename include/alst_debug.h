/*
 * alst_debug.h -- benchmarking and testing aids of libalst.  None of them is part of the method
 * (no counterpart in the paper) and no product code needs them: the timers serve the benchmark,
 * the block mapping and the matrix-instruction rate serve the tests and the roofline context.
 */
#ifndef ALST_DEBUG_H
#define ALST_DEBUG_H

#include "alst.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Benchmarking aid (no counterpart in the paper).  While enabled, every launch of a block GEMM and
 * each group of small kernels between them is bracketed by a pair of HIP events on the launch
 * stream.  alst_profile_read() waits for the recorded events, writes per kind the summed
 * milliseconds and the number of spans into the HOST arrays ms_total[8] and launches[8], and
 * forgets the spans.  Kinds: 0 logits GEMM, 1 dHidden GEMM, 2 dW GEMM, 3 the small kernels of a
 * cross-entropy tile; 4 the projection GEMMs of the tiled MLP (alst_mlp.h), 5 its weight-gradient
 * GEMMs, 6 its small kernels; 7 unused.  The recorded spans are process-wide state behind a lock:
 * calls from several host threads are safe, and their spans land in one list.
 */
int alst_profile_enable(int on);
int alst_profile_read(double* ms_total, int64_t* launches);

/*
 * Testing aid (no counterpart in the paper; host arithmetic only, no device is touched).  The block
 * GEMM launches deal their workgroups round-robin to the 8 XCDs of the chip and give the 32
 * workgroups resident on one XCD a compact patch of output blocks; a launch may hold several
 * products ("parts") whose patches are numbered through.  For a launch of `parts` products of
 * tiles_r x tiles_c blocks this returns the number of workgroups and writes, for workgroup `bid`,
 * the part and block it computes (part = -1: the workgroup leaves at once), evaluated with the
 * same functions the kernels use.  A negative return value is minus an alst_status.
 */
int alst_debug_block_tile(int tiles_r, int tiles_c, int parts, int bid, int* part, int* tr, int* tc);

/*
 * Benchmarking aid (no counterpart in the paper): the sustained rate, in TFLOP/s, of the bf16
 * matrix instructions the block GEMMs are built on, measured on the current device with a loop that
 * touches no memory (one wavefront per SIMD of every compute unit, iters * 2^21 flop each).
 * It is the ceiling the GEMM kernels can be compared with besides the published peak: the clock
 * under matrix load depends on the power drawn, hence on the operand bits and the instruction form.
 * data bit 0: 0 = small-integer operands, 1 = random operands in [-1, 1); data bit 1: 0 =
 * v_mfma_f32_32x32x16_bf16 (the cores with a k-major operand), 1 = v_mfma_f32_16x16x32_bf16 (the
 * k-contiguous core).  scratch: device, 256 * 256 floats, overwritten; tflops: HOST double.
 * 1 <= iters <= 2^22; any other data is ALST_ERR_SHAPE.  Synchronises `stream`.
 */
int alst_debug_mfma_rate(int data, int iters, float* scratch, double* tflops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ALST_DEBUG_H */
