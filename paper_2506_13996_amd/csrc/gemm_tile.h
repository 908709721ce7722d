// Block-tile bf16 MFMA contraction for gfx950, shared by the three GEMMs of the tiled LM-head +
// cross-entropy path (logits of a sequence tile, dHidden of the tile, dW accumulation).
//
//     D[r][c] = sum_k X[r][k] * Y[c][k]          X, Y bf16 with k contiguous, fp32 accumulation
//
// One workgroup of 512 threads (8 wavefronts, 2 per SIMD) owns a 256 (r) x 256 (c) block of D and
// walks k in steps of 64.  Operand tiles go global -> registers -> LDS (16-byte chunks, XOR
// swizzled so that both the 16-byte stores and the MFMA operand reads are bank-conflict free) and
// are double buffered: the global loads of step k+1 are in flight while step k is multiplied.
// Wavefront w owns the 64 (r) x 128 (c) sub-block (w & 3, w >> 2) as 2 x 4 MFMA 32x32x16 tiles.
// The c index is the MFMA row (register) dimension and r the MFMA column (lane) dimension, so a
// lane holds, for one r, runs of 4 consecutive c: reductions over c stay mostly inside a lane and
// stores along c are vector stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace alst {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kBlockR = 256;          // rows of X per block (MFMA lane dimension)
constexpr int kBlockC = 256;          // rows of Y per block (MFMA register dimension)
constexpr int kBlockK = 64;           // k per main-loop step
constexpr int kThreads = 512;
constexpr int kWaveR = 64, kWaveC = 128;
constexpr int kMT = 4;                // 32-wide c tiles per wavefront
constexpr int kNT = 2;                // 32-wide r tiles per wavefront
constexpr int kTileBytes = kBlockR * kBlockK * 2;       // one operand tile in LDS
constexpr int kLdsBytes = 4 * kTileBytes;               // X, Y, two stages each

// Where the calling lane's accumulators sit inside the block.
struct LanePos {
    int lane, half, l31, wr, wc;
    __device__ __forceinline__ LanePos() {
        const int tid = threadIdx.x;
        lane = tid & 63;
        half = lane >> 5;
        l31 = lane & 31;
        const int wave = tid >> 6;
        wr = wave & 3;
        wc = wave >> 2;
    }
    // row of X (r index inside the block) of accumulator tile nt
    __device__ __forceinline__ int r(int nt) const { return wr * kWaveR + nt * 32 + l31; }
    // first of the 4 consecutive c held in registers 4q..4q+3 of accumulator tile mt
    __device__ __forceinline__ int c(int mt, int q) const {
        return wc * kWaveC + mt * 32 + q * 8 + half * 4;
    }
};

// XCD-aware block -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs (each with its
// own L2); the 32 workgroups that are resident together on one XCD get a compact PR x PC patch of
// tiles so that they share operand rows through that L2.  Returns false for padding blocks.
template <int PR, int PC>
__device__ __forceinline__ bool tile_of_block(int bid, int tiles_r, int tiles_c, int& tr, int& tc) {
    constexpr int kPatch = PR * PC;
    const int xcd = bid & 7;
    const int slot = bid >> 3;
    const int p = slot / kPatch, w = slot % kPatch;
    const int patches_r = (tiles_r + PR - 1) / PR;
    const int patches_c = (tiles_c + PC - 1) / PC;
    const int P = p * 8 + xcd;
    if (P >= patches_r * patches_c) return false;
    tr = (P % patches_r) * PR + (w % PR);
    tc = (P / patches_r) * PC + (w / PR);
    return tr < tiles_r && tc < tiles_c;
}

template <int PR, int PC>
inline int grid_for_tiles(int tiles_r, int tiles_c) {
    const int patches = ((tiles_r + PR - 1) / PR) * ((tiles_c + PC - 1) / PC);
    return ((patches + 7) / 8) * 8 * PR * PC;
}

// acc[mt][nt] += X-block(r0) * Y-block(c0)^T over all of K.
// GUARD = false requires r0 + 256 <= rows_x, c0 + 256 <= rows_y and K % 64 == 0.
// GUARD = true zero-fills rows beyond rows_x / rows_y and k beyond K (K % 8 == 0 required).
template <bool GUARD>
__device__ __forceinline__ void block_gemm(const uint16_t* __restrict__ X, int64_t ldx, int rows_x,
                                           const uint16_t* __restrict__ Y, int64_t ldy, int rows_y,
                                           int K, int r0, int c0, unsigned char* smem,
                                           f32x16_t (&acc)[kMT][kNT]) {
    const int tid = threadIdx.x;
    const LanePos lp;
    const int lrow = tid >> 3;      // 0..63, row inside a 64-row slab of the operand tile
    const int kc = tid & 7;         // 16-byte chunk along k

    const uint16_t* xp[4];
    const uint16_t* yp[4];
    bool xv[4], yv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int gx = r0 + lrow + 64 * j, gy = c0 + lrow + 64 * j;
        xv[j] = !GUARD || gx < rows_x;
        yv[j] = !GUARD || gy < rows_y;
        xp[j] = X + (int64_t)(xv[j] ? gx : 0) * ldx + kc * 8;
        yp[j] = Y + (int64_t)(yv[j] ? gy : 0) * ldy + kc * 8;
    }
    const int wofs = (lrow * 8 + (kc ^ (lrow & 7))) * 16;          // + j * 64 rows * 128 B
    int rofs[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) rofs[s] = ((2 * s + lp.half) ^ (lp.lane & 7)) * 16;
    const int xbase = (lp.wr * kWaveR + lp.l31) * 128;
    const int ybase = (lp.wc * kWaveC + lp.l31) * 128;

    unsigned char* const Xs = smem;
    unsigned char* const Ys = smem + 2 * kTileBytes;

    u32x4_t xg[4], yg[4];
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};

    auto load_global = [&](int kt) {
        const int koff = kt * kBlockK;
        const bool kok = !GUARD || (koff + kc * 8 + 8 <= K);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            xg[j] = (xv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(xp[j] + koff) : zero4;
            yg[j] = (yv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(yp[j] + koff) : zero4;
        }
    };
    auto store_lds = [&](int stage) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *reinterpret_cast<u32x4_t*>(Xs + stage * kTileBytes + wofs + j * 8192) = xg[j];
            *reinterpret_cast<u32x4_t*>(Ys + stage * kTileBytes + wofs + j * 8192) = yg[j];
        }
    };

    const int KT = (K + kBlockK - 1) / kBlockK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) load_global(kt + 1);
        const unsigned char* xs = Xs + cur * kTileBytes + xbase;
        const unsigned char* ys = Ys + cur * kTileBytes + ybase;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8_t yf[kMT], xf[kNT];
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
                yf[mt] = *reinterpret_cast<const bf16x8_t*>(ys + mt * 4096 + rofs[s]);
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
                xf[nt] = *reinterpret_cast<const bf16x8_t*>(xs + nt * 4096 + rofs[s]);
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                for (int nt = 0; nt < kNT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yf[mt], xf[nt],
                                                                          acc[mt][nt], 0, 0, 0);
        }
        if (more) store_lds(cur ^ 1);
        __syncthreads();
    }
}

}  // namespace alst
