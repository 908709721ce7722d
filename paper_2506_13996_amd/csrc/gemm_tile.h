// Block-tile bf16 MFMA contraction for gfx950, shared by every GEMM of the library: the tiled
// LM-head + cross-entropy path (logits of a sequence tile, dHidden of the tile, dW accumulation),
// the tiled MLP and the tiled linear layer.
//
// One workgroup owns a 256 (r) x 256 (c) block of D and walks k in steps of 64 through two LDS
// stages.  The c index is the MFMA row (register) dimension and r the MFMA column (lane)
// dimension, so a lane holds, for one r, runs of 4 consecutive c: reductions over c stay mostly
// inside a lane and stores along c are vector stores.  The DMA cores multiply with
// v_mfma_f32_16x16x32_bf16 (accumulator tiles of 16 x 16, 4 registers per lane), the
// register-staged cores with v_mfma_f32_32x32x16_bf16 (32 x 32, 16 registers): on random operands
// the 16 x 16 form draws less power per flop (a register-resident loop sustains 1.89 against
// 1.80 PFLOP/s) and the same block GEMM runs 5.5 - 7.5 % faster with it.  The kernels' epilogues
// are written against the layout description every core carries (Lane, kTile, kRuns, kGroups).
//
// An operand is either k-contiguous (a matrix [rows][k]) or k-major (a matrix [k][columns], the
// block taking 256 of its columns).  Three combinations occur:
//     D[r][c] = sum_k X[r][k] * Y[c][k]     both k-contiguous: logits, forward projections
//     D[r][c] = sum_k X[r][k] * Y[k][c]     "mixed": a product with a weight matrix over its row
//                                           index (dH = dZ W, da = dy Wd, dx = dg Wg + du Wu)
//     D[r][c] = sum_k X[k][r] * Y[k][c]     both k-major: the weight-gradient products, whose k is
//                                           the token row
// so that every operand is read from memory as it is and nothing is ever transposed.
//
// Two families of cores with the same accumulator interface, each in the three layouts:
//   DirectCore, MixedCore, KMajorCore
//               4 wavefronts (one per SIMD), 128 x 128 per wavefront, operands DMA'd straight from
//               global memory into LDS (global_load_lds_dwordx4), MFMA operands of the two
//               k-slices of a step held in registers, one barrier in the middle of a k-step so
//               that the next stage's first operands are read while the second half is
//               multiplied.  A k-major tile lands in LDS as 64 k-rows and the MFMA operands are
//               formed by the transposing LDS read (ds_read_b64_tr_b16).  No bounds checks in the
//               DMA path: every extent block-aligned (see gemm for the exceptions).
//   StagedCore, StagedMixedCore, StagedKMajorCore
//               8 wavefronts, 64 x 128 per wavefront, operands staged through registers with
//               zero fill outside the matrices: the fallback for ragged shapes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace alst {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef short i16x8_t __attribute__((ext_vector_type(8)));

constexpr int kBlockR = 256;          // rows of X per block (MFMA lane dimension)
constexpr int kBlockC = 256;          // rows of Y per block (MFMA register dimension)
constexpr int kBlockK = 64;           // k per main-loop step
constexpr int kGroupC = 128;          // c extent one wavefront covers (all cores)
constexpr int kTileBytes = kBlockR * kBlockK * 2;       // one operand tile in LDS (32 KB)
constexpr int kStageBytes = 4 * kTileBytes;             // X, Y, two stages each (128 KB)
constexpr int kLdsBytes = kStageBytes + 1024;           // + landing area of the L2 warm-up loads
constexpr int kWarmAhead = 3;                           // k-steps between warm-up and DMA of a line

// XCD-aware block -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs (each with its
// own L2); the 32 workgroups that are resident together on one XCD get a compact PR x PC patch of
// output blocks so that they share operand tiles through that L2.  The patch shape is chosen per
// launch, and a launch may hold several products ("parts"): the patches of all parts are numbered
// through, and patch P goes to XCD P % 8, so the XCDs stay evenly loaded whatever the number of
// patches of one part is.
struct PatchGrid {
    int tiles_r, tiles_c;      // output blocks of one part
    int PR, PC;                // patch shape, PR * PC = 32
    __host__ __device__ int patches_r() const { return (tiles_r + PR - 1) / PR; }
    // (int: the launches are checked to fit a one-dimensional grid before any kernel sees this)
    __host__ __device__ int patches() const { return patches_r() * ((tiles_c + PC - 1) / PC); }
    // for the host-side sizing, which also meets shapes no launch can hold
    int64_t patches64() const { return (int64_t)patches_r() * ((tiles_c + PC - 1) / PC); }
};

// Patch shape: 4 x 8 (12 operand tiles per k-step for 32 blocks), unless 8 x 4 or one of the
// flat shapes 2 x 16, 16 x 2 (18 tiles per k-step) pads so much less that it needs under 9/10 of
// the patches.
inline PatchGrid choose_patches(int tiles_r, int tiles_c) {
    const int shapes[4][2] = {{4, 8}, {8, 4}, {2, 16}, {16, 2}};
    PatchGrid best = {tiles_r, tiles_c, 4, 8};
    for (int i = 1; i < 4; ++i) {
        const PatchGrid g = {tiles_r, tiles_c, shapes[i][0], shapes[i][1]};
        if (10 * g.patches64() < 9 * best.patches64()) best = g;
    }
    return best;
}

inline int grid_for_patches(int64_t patches) { return (int)(((patches + 7) / 8) * 8 * 32); }

// Workgroup -> (global patch number, position inside the patch).
__host__ __device__ __forceinline__ void patch_of_block(int bid, int& P, int& w) {
    const int slot = bid >> 3;
    P = (slot >> 5) * 8 + (bid & 7);
    w = slot & 31;
}

// Block (tr, tc) of position w in local patch P of g; false if the patch sticks out there.
__host__ __device__ __forceinline__ bool tile_in_patch(const PatchGrid& g, int P, int w, int& tr,
                                                       int& tc) {
    const int pr = g.patches_r();
    tr = (P % pr) * g.PR + (w % g.PR);
    tc = (P / pr) * g.PC + (w / g.PR);
    return tr < g.tiles_r && tc < g.tiles_c;
}

// Gated pair of Y operands: with Y2 given, the 256 Y rows of the block at c0 are four runs of 64
// rows, run q = rows c0 / 2 + (q / 2) * 64 .. + 63 of Y (q even) or of Y2 (q odd): the 128 rows of
// a wavefront are 64 rows of Y followed by the same 64 rows of Y2, so a lane that holds the
// product with row j of Y in accumulator tile mt holds the one with row j of Y2 in the tile 64 rows on
// (mt + 2 for 32-row tiles, mt + 4 for 16-row tiles).
// br = row inside the block; valid = the source row exists (the pointer is then usable anyway).
__device__ __forceinline__ const uint16_t* paired_row(const uint16_t* Y, const uint16_t* Y2,
                                                      int64_t ldy, int c0, int br, int rows_y,
                                                      bool& valid) {
    const int run = br >> 6;
    const int src = (c0 >> 1) + (run >> 1) * 64 + (br & 63);
    valid = src < rows_y;
    return ((run & 1) ? Y2 : Y) + (int64_t)(valid ? src : 0) * ldy;
}

// L2 warm-up.  The blocks of a patch that share an operand tile walk k in step, so each of them
// would meet every line of the tile as an L2 miss at the same moment.  Instead the sharers split
// the tile's rows between them and each touches one dword per line of its share kWarmAhead
// k-steps before the DMA needs it: the miss latency is paid early and once, and the sixteen DMA
// instructions of a k-step find their lines in L2.  Returns this lane's row of X or Y (the
// pointer to its first element); every lane gets a valid row, surplus lanes repeat one.  PR x PC
// is the launch's patch shape (2 x 16, 4 x 8, 8 x 4 or 16 x 2).
__device__ __forceinline__ const uint16_t* warm_row(int PR, int PC, const uint16_t* X, int64_t ldx,
                                                    int r0, int tr, const uint16_t* Y, int64_t ldy,
                                                    int c0, int tc, const uint16_t* Y2 = nullptr,
                                                    int rows_y = 0x7fffffff) {
    const int nx = kBlockR / PC, ny = kBlockC / PR, total = nx + ny, per = (total + 3) / 4;   // per <= 36
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int l = w * per + (lane < per ? lane : per - 1);
    if (l > total - 1) l = total - 1;
    if (l < nx) return X + (int64_t)(r0 + (tc % PC) * nx + l) * ldx;
    if (Y2) {
        bool valid;
        return paired_row(Y, Y2, ldy, c0, (tr % PR) * ny + (l - nx), rows_y, valid);
    }
    const int row = c0 + (tr % PR) * ny + (l - nx);
    return Y + (int64_t)(row < rows_y ? row : rows_y - 1) * ldy;      // as the DMA: clamped to Y
}

// The same for k-major operands X[k][ldx], Y[k][ldy]: the 64 k-rows x 512 bytes of a k-step's tile
// are 256 lines, line L = (k-row L / 4, 128-byte piece L % 4).  `step` = elements between the
// lane's line in one k-step and the next.
__device__ __forceinline__ const uint16_t* warm_line_kmajor(int PR, int PC, const uint16_t* X,
                                                            int64_t ldx, int r0, int tr,
                                                            const uint16_t* Y, int64_t ldy, int c0,
                                                            int tc, int64_t& step,
                                                            int cols_x = 0x7fffffff,
                                                            int cols_y = 0x7fffffff) {
    const int nx = kBlockR / PC, ny = kBlockC / PR, total = nx + ny, per = (total + 3) / 4;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int l = w * per + (lane < per ? lane : per - 1);
    if (l > total - 1) l = total - 1;
    if (l < nx) {
        const int L = (tc % PC) * nx + l;
        step = ldx * kBlockK;
        const int col = r0 + (L & 3) * 64;
        return X + (int64_t)(L >> 2) * ldx + (col < cols_x ? col : cols_x - 8);
    }
    const int L = (tr % PR) * ny + (l - nx);
    step = ldy * kBlockK;
    const int col = c0 + (L & 3) * 64;
    return Y + (int64_t)(L >> 2) * ldy + (col < cols_y ? col : cols_y - 8);
}

// X k-contiguous (its lines are rows), Y k-major.
__device__ __forceinline__ const uint16_t* warm_line_mixed(int PR, int PC, const uint16_t* X,
                                                           int64_t ldx, int r0, int tr,
                                                           const uint16_t* Y, int64_t ldy, int c0,
                                                           int tc, int64_t& step,
                                                           int cols_y = 0x7fffffff,
                                                           int krows_y = 0x7fffffff) {
    const int nx = kBlockR / PC, ny = kBlockC / PR, total = nx + ny, per = (total + 3) / 4;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int l = w * per + (lane < per ? lane : per - 1);
    if (l > total - 1) l = total - 1;
    if (l < nx) {
        step = kBlockK;
        return X + (int64_t)(r0 + (tc % PC) * nx + l) * ldx;
    }
    const int L = (tr % PR) * ny + (l - nx);
    step = ldy * kBlockK;
    const int col = c0 + (L & 3) * 64;
    const int krow = (L >> 2) < krows_y ? (L >> 2) : krows_y - 1;
    return Y + (int64_t)krow * ldy + (col < cols_y ? col : cols_y - 8);
}

// ---------------------------------------------------------------------------------------------
// StagedCore: 8 wavefronts, register staging, optional bounds checks
// ---------------------------------------------------------------------------------------------
// k-major LDS tiles (both cores): an LDS row is one k-row of 512 bytes = 8 granules of 64 bytes
// (32 r or c each); granule g of k-row k lives at granule slot g ^ kswz(k).  One transposing read
// covers k-rows {R .. R+3, R+8 .. R+11} (R % 4 == 0) at one granule: 8 different slots.
__device__ __forceinline__ int kswz(int k) { return (k & 3) | (((k >> 3) & 1) << 2); }

// MFMA operand (8 k of one column per lane) from a k-major tile: two transposing reads.  In each,
// the 16 lanes of a quarter wave address 4 k-rows x 4 pieces of 8 bytes and lane i of the quarter
// receives the 4 k of column i.  `at`: the lane's address for the first 4 k-rows; the next 4
// k-rows are 2048 bytes on.
__device__ __forceinline__ bf16x8_t read_kmajor(const unsigned char* at) {
    typedef __attribute__((address_space(3))) i16x4_t* tptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    unsigned char* const p = const_cast<unsigned char*>(at);
    const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tptr_t)(lptr_t)p);
    const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tptr_t)(lptr_t)(p + 2048));
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// The lane's byte offset inside a k-major tile for granule `gran` (MFMA lane l: column l % 32 of
// the granule, k = 8 (l / 32) .. + 7 of a 16-row slice; add 8192 per slice).
__device__ __forceinline__ int kmajor_lane_offset(int lane, int gran) {
    const int sl = lane & 15, b1 = (lane >> 4) & 1, half = lane >> 5;
    const int f = (sl >> 2) | (half << 2);                   // kswz of the lane's k-rows
    return (8 * half + (sl >> 2)) * 512 + ((gran ^ f) * 64) + b1 * 32 + (sl & 3) * 8;
}

// Values that are the same in every lane of a wavefront, said so to the compiler (it then keeps
// them in scalar registers and branches on them without masking lanes).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
template <class T>
__device__ __forceinline__ const T* uniform(const T* p) {
    return reinterpret_cast<const T*>(uniform((int64_t)reinterpret_cast<uintptr_t>(p)));
}

// Global -> LDS DMA: each lane's BYTES (16 or 4) land at lds + lane * BYTES; `lds` must be uniform
// over the wavefront.
template <int BYTES>
__device__ __forceinline__ void dma_to_lds(const void* g, unsigned char* lds) {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    static_assert(BYTES == 16 || BYTES == 4, "one or four dwords per lane");
    if (BYTES == 16) __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)lds, 16, 0, 0);
    else __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)lds, 4, 0, 0);
}

// Combines a value over the lane groups of a wavefront that hold the same r (lanes l, l ^ 16, l ^ 32,
// l ^ 48 for 16 x 16 tiles; l, l ^ 32 for 32 x 32 tiles): every lane gets the result.
template <int GROUPS>
__device__ __forceinline__ float groups_max(float v) {
    if (GROUPS == 4) v = fmaxf(v, __shfl_xor(v, 16));
    return fmaxf(v, __shfl_xor(v, 32));
}
template <int GROUPS>
__device__ __forceinline__ float groups_sum(float v) {
    if (GROUPS == 4) v += __shfl_xor(v, 16);
    return v + __shfl_xor(v, 32);
}

// XK / YK: that operand is k-major.
template <bool XK, bool YK>
struct StagedCoreT {
    static constexpr int kThreads = 512;
    static constexpr int kMT = 4;     // 32-wide c tiles per wavefront
    static constexpr int kNT = 2;     // 32-wide r tiles per wavefront
    static constexpr bool kCanGuard = true;
    // accumulator layout: tiles of kTile x kTile; a lane holds kRuns runs of 4 consecutive c per
    // tile; kGroups lane groups hold the same r
    typedef f32x16_t acc_t;
    static constexpr int kTile = 32, kRuns = 4, kGroups = 2;

    // Where the calling lane's accumulators sit inside the block.
    struct Lane {
        int lane, grp, lrow, wr, wc;
        __device__ __forceinline__ Lane() {
            const int tid = threadIdx.x;
            lane = tid & 63;
            grp = lane >> 5;
            lrow = lane & 31;
            const int wave = tid >> 6;
            wr = wave & 3;
            wc = wave >> 2;
        }
        // row of X (r index inside the block) of accumulator tile nt
        __device__ __forceinline__ int r(int nt) const { return wr * 64 + nt * 32 + lrow; }
        // first of the 32 rows of accumulator tile nt that this wavefront holds
        __device__ __forceinline__ int rbase(int nt) const { return wr * 64 + nt * 32; }
        // first of the 4 consecutive c held in registers 4q..4q+3 of accumulator tile mt: inside
        // the wavefront's 128 columns (cw) and inside the block (c)
        __device__ __forceinline__ int cw(int mt, int q) const { return mt * 32 + q * 8 + grp * 4; }
        __device__ __forceinline__ int c(int mt, int q) const { return wc * kGroupC + cw(mt, q); }
    };

    // acc[mt][nt] += X-block(r0) * Y-block(c0)^T over all of K.
    // GUARD = false requires r0 + 256 <= rows_x, c0 + 256 <= rows_y and K % 64 == 0.
    // GUARD = true zero-fills outside the operands.  A k-contiguous operand is [rows][ld] with
    // its rows beyond rows_x / rows_y and its k beyond K read as zero (K % 8 == 0 required); a
    // k-major operand is [K][ld], the block takes its columns r0 .. r0 + 255 (c0 ..), rows_x
    // (rows_y) is its number of columns (a multiple of 8), and any K goes.  K_y, if given, is the
    // k extent of Y where that is shorter than the loop's K (X zero-padded along k, Y not).
    // Y2: gated pair, see paired_row (k-contiguous Y only).
    template <bool GUARD>
    static __device__ __forceinline__ void gemm(const uint16_t* __restrict__ X, int64_t ldx,
                                                int rows_x, const uint16_t* __restrict__ Y,
                                                int64_t ldy, int rows_y, int K, int r0, int c0,
                                                unsigned char* smem, f32x16_t (&acc)[kMT][kNT],
                                                const uint16_t* /*warm*/ = nullptr,
                                                int64_t /*warm_stride*/ = 0,
                                                const uint16_t* Y2 = nullptr, int K_y = -1) {
        const int tid = threadIdx.x;
        const Lane lp;
        if (K_y < 0) K_y = K;
        // k-contiguous operand: thread -> (row tid / 8 inside a 64-row slab of the tile, 16-byte
        // chunk tid % 8 along k), slab j = 0..3;  k-major operand: thread -> (k-row tid / 32 + 16 j,
        // 16-byte chunk of 8 columns tid % 32)
        const int xrow = XK ? (tid >> 5) : (tid >> 3), xch = XK ? (tid & 31) : (tid & 7);
        const int yrow = YK ? (tid >> 5) : (tid >> 3), ych = YK ? (tid & 31) : (tid & 7);

        const uint16_t* xp[4];
        const uint16_t* yp[4];
        bool xv[4], yv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (XK) {
                xv[j] = !GUARD || r0 + xch * 8 < rows_x;
                xp[j] = X + (int64_t)(xrow + 16 * j) * ldx + (xv[j] ? r0 + xch * 8 : 0);
            } else {
                const int gx = r0 + xrow + 64 * j;
                xv[j] = !GUARD || gx < rows_x;
                xp[j] = X + (int64_t)(xv[j] ? gx : 0) * ldx + xch * 8;
            }
            if (YK) {
                yv[j] = !GUARD || c0 + ych * 8 < rows_y;
                yp[j] = Y + (int64_t)(yrow + 16 * j) * ldy + (yv[j] ? c0 + ych * 8 : 0);
            } else if (Y2) {
                bool valid;
                yp[j] = paired_row(Y, Y2, ldy, c0, yrow + 64 * j, rows_y, valid) + ych * 8;
                yv[j] = !GUARD || valid;
            } else {
                const int gy = c0 + yrow + 64 * j;
                yv[j] = !GUARD || gy < rows_y;
                yp[j] = Y + (int64_t)(yv[j] ? gy : 0) * ldy + ych * 8;
            }
        }
        // k-contiguous tile: 16-byte chunk kc of row `row` lives at chunk slot kc ^ (row & 7) of
        // its 128-byte row (+ j * 64 rows * 128 B);  k-major tile: see kswz (+ j * 16 k-rows * 512 B)
        const int xwofs = XK ? xrow * 512 + ((xch ^ (kswz(xrow) << 2)) * 16)
                             : (xrow * 8 + (xch ^ (xrow & 7))) * 16;
        const int ywofs = YK ? yrow * 512 + ((ych ^ (kswz(yrow) << 2)) * 16)
                             : (yrow * 8 + (ych ^ (yrow & 7))) * 16;
        int rofs[4], xofs[kNT], yofs[kMT];
#pragma unroll
        for (int s = 0; s < 4; ++s) rofs[s] = ((2 * s + lp.grp) ^ (lp.lane & 7)) * 16;
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt) xofs[nt] = kmajor_lane_offset(lp.lane, lp.wr * kNT + nt);
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt) yofs[mt] = kmajor_lane_offset(lp.lane, lp.wc * kMT + mt);
        const int xbase = (lp.wr * 64 + lp.lrow) * 128;
        const int ybase = (lp.wc * kGroupC + lp.lrow) * 128;

        unsigned char* const Xs = smem;
        unsigned char* const Ys = smem + 2 * kTileBytes;

        u32x4_t xg[4], yg[4];
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};

        auto load_global = [&](int kt) {
            const int koff = kt * kBlockK;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (XK) {
                    const bool kok = !GUARD || (koff + xrow + 16 * j < K);
                    xg[j] = (xv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(xp[j] + (int64_t)koff * ldx) : zero4;
                } else {
                    const bool kok = !GUARD || (koff + xch * 8 + 8 <= K);
                    xg[j] = (xv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(xp[j] + koff) : zero4;
                }
                if (YK) {
                    const bool kok = !GUARD || (koff + yrow + 16 * j < K_y);
                    yg[j] = (yv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(yp[j] + (int64_t)koff * ldy) : zero4;
                } else {
                    const bool kok = !GUARD || (koff + ych * 8 + 8 <= K_y);
                    yg[j] = (yv[j] && kok) ? *reinterpret_cast<const u32x4_t*>(yp[j] + koff) : zero4;
                }
            }
        };
        auto store_lds = [&](int stage) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                *reinterpret_cast<u32x4_t*>(Xs + stage * kTileBytes + xwofs + j * 8192) = xg[j];
                *reinterpret_cast<u32x4_t*>(Ys + stage * kTileBytes + ywofs + j * 8192) = yg[j];
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
                    yf[mt] = YK ? read_kmajor(Ys + cur * kTileBytes + yofs[mt] + s * 8192)
                                : *reinterpret_cast<const bf16x8_t*>(ys + mt * 4096 + rofs[s]);
#pragma unroll
                for (int nt = 0; nt < kNT; ++nt)
                    xf[nt] = XK ? read_kmajor(Xs + cur * kTileBytes + xofs[nt] + s * 8192)
                                : *reinterpret_cast<const bf16x8_t*>(xs + nt * 4096 + rofs[s]);
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
};
typedef StagedCoreT<false, false> StagedCore;
typedef StagedCoreT<true, true> StagedKMajorCore;
typedef StagedCoreT<false, true> StagedMixedCore;

// ---------------------------------------------------------------------------------------------
// KMajorDirectT: the DMA core for a k-major Y (and, with XK, a k-major X): v_mfma_f32_32x32x16_bf16
// ---------------------------------------------------------------------------------------------
// Same pipeline as DirectCore below on 32 x 32 accumulator tiles.  Measured on the dHidden and dW
// GEMMs the 16 x 16 x 32 form gains nothing over this one when operands come through the
// transposing reads, and its register allocation breaks down for two k-major operands.
// XK: X is k-major too.
template <bool XK>
struct KMajorDirectT {
    static constexpr bool YK = true;
    static constexpr int kThreads = 256;
    static constexpr int kMT = 4;     // 32-wide c tiles per wavefront
    static constexpr int kNT = 4;     // 32-wide r tiles per wavefront
    static constexpr bool kCanGuard = false;
    typedef f32x16_t acc_t;
    static constexpr int kTile = 32, kRuns = 4, kGroups = 2;

    struct Lane {
        int lane, grp, lrow, wr, wc;
        __device__ __forceinline__ Lane() {
            const int tid = threadIdx.x;
            lane = tid & 63;
            grp = lane >> 5;
            lrow = lane & 31;
            const int wave = tid >> 6;
            wr = wave & 1;
            wc = wave >> 1;
        }
        __device__ __forceinline__ int r(int nt) const { return wr * 128 + nt * 32 + lrow; }
        __device__ __forceinline__ int rbase(int nt) const { return wr * 128 + nt * 32; }
        __device__ __forceinline__ int cw(int mt, int q) const { return mt * 32 + q * 8 + grp * 4; }
        __device__ __forceinline__ int c(int mt, int q) const { return wc * kGroupC + cw(mt, q); }
    };

    // LDS row = 128 bytes = 8 chunks of 16 bytes; chunk kc of row `row` lives at slot
    // kc ^ ((row >> 1) & 7): sixteen consecutive rows at one kc then cover all 64 banks once.
    static __device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

    // Requires K % 64 == 0, K >= 64, 16-byte aligned rows, and a k-contiguous X with r0 + 256 <= its
    // rows.  GUARD must be false.  Y is [K][ldy] and the block takes its columns c0 .. c0 + 255; a
    // k-major X is [K][ldx], columns r0 .. r0 + 255.  A k-major operand with rows_x / rows_y
    // columns (a multiple of 8) may end inside the block: it is read from its last 8 columns in
    // place of those beyond (a hidden size that is not a multiple of the block width), finite data
    // of the operand, and the caller discards the accumulator rows / columns that lie outside.
    // With YTAIL (k-contiguous X only): K_y (if >= 0 and < K) is the k extent Y has when X is
    // zero-padded along k beyond it (W in dH = dZ W for a vocabulary that is not whole k-steps):
    // the k-rows of the last step that Y lacks are read from its last row and meet zeros of X.
    // warm_stride = elements between the lane's warm-up line of one k-step and the next.
    template <bool GUARD, bool YTAIL = false>
    static __device__ __forceinline__ void gemm(const uint16_t* __restrict__ X, int64_t ldx,
                                                int rows_x, const uint16_t* __restrict__ Y,
                                                int64_t ldy, int rows_y, int K, int r0, int c0,
                                                unsigned char* smem, acc_t (&acc)[kMT][kNT],
                                                const uint16_t* warm, int64_t warm_stride = kBlockK,
                                                const uint16_t* /*Y2*/ = nullptr, int K_y = -1) {
        static_assert(!GUARD, "the DMA cores have no bounds checks");
        const int tid = threadIdx.x, lane = tid & 63;
        const int w = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave id, provably uniform
        const int wr = w & 1, wc = w >> 1;
        const int l31 = lane & 31, half = lane >> 5;

        // One DMA instruction moves 8 rows x 128 bytes: lane -> (row = lane / 8, LDS chunk slot =
        // lane % 8); the lane fetches the global chunk that belongs in its slot.  Wave w owns rows
        // [64 w, 64 w + 64) of both operand tiles: 8 instructions per operand per k-step.
        // k-major: one DMA instruction moves 2 k-rows x 512 bytes: lane -> (k-row = lane / 32, chunk
        // slot = lane % 32); wave w owns k-rows [16 w, 16 w + 16) of the tile.
        const int lr = lane >> 3, pc = lane & 7;
        const uint16_t* xg[8];
        const uint16_t* yg[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int krow = w * 16 + q * 2 + (lane >> 5);
            const int ch = (lane & 31) ^ (kswz(krow) << 2);
            const int row = (w * 8 + q) * 8 + lr;
            const int kc = pc ^ swz(row);
            // (the clamps: see the comment of this function)
            if (XK) xg[q] = X + (int64_t)krow * ldx + (r0 + ch * 8 < rows_x ? r0 + ch * 8 : rows_x - 8);
            else xg[q] = X + (int64_t)(r0 + row) * ldx + kc * 8;
            yg[q] = Y + (int64_t)krow * ldy + (c0 + ch * 8 < rows_y ? c0 + ch * 8 : rows_y - 8);
        }
        // elements from one k-step's tile to the next
        const int64_t xstep = XK ? ldx * kBlockK : kBlockK, ystep = ldy * kBlockK;
        // Y shorter than the loop's K (X zero-padded along k beyond K_y): the lane's sources in the
        // last k-step, the k-rows Y lacks read from its last row.
        constexpr bool kTail = YTAIL && !XK;
        const int KT_ = K / kBlockK;
        const bool ytail = kTail && K_y >= 0 && K_y < K;
        const uint16_t* yg_tail[8];
        if (kTail) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int krow = (KT_ - 1) * kBlockK + w * 16 + q * 2 + (lane >> 5);
                const int ch = (lane & 31) ^ (kswz(krow) << 2);
                const int kr = ytail && krow >= K_y ? K_y - 1 : krow;
                yg_tail[q] = Y + (int64_t)kr * ldy + (c0 + ch * 8 < rows_y ? c0 + ch * 8 : rows_y - 8);
            }
        }
        auto ysrc = [&](int q, int kt) -> const uint16_t* {
            if (kTail) return (ytail && kt == KT_ - 1) ? yg_tail[q] : yg[q] + kt * ystep;
            return yg[q] + kt * ystep;
        };
        auto issue_loads = [&](int stage, int kt) {
            unsigned char* xs = smem + stage * kTileBytes + w * 8192;
            unsigned char* ys = smem + 2 * kTileBytes + stage * kTileBytes + w * 8192;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                dma_to_lds<16>(xg[q] + kt * xstep, xs + q * 1024);
                dma_to_lds<16>(ysrc(q, kt), ys + q * 1024);
            }
        };

        // Operand reads.  k-contiguous tiles: one 16-byte read per operand.  k-major: read_kmajor.
        int rofs[4], xofs[4], yofs[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            rofs[s] = ((2 * s + half) ^ swz(l31)) * 16;
            xofs[s] = kmajor_lane_offset(lane, wr * 4 + s);      // s = accumulator tile here
            yofs[s] = 2 * kTileBytes + kmajor_lane_offset(lane, wc * 4 + s);
        }
        const int xbase = (wr * 128 + l31) * 128;

        // MFMA operands of the four k-slices of a step: fy[s][t], fx[s][t] for slice s.
        bf16x8_t fy[4][4], fx[4][4];
        // item 0..3: the Y operand of accumulator row t = item, 4..7: the X operand of column t
        auto read_item = [&](int stage, int s, int item) {
            const unsigned char* base = smem + stage * kTileBytes;
            if (item < 4)
                fy[s][item] = read_kmajor(base + yofs[item] + s * 8192);
            else
                fx[s][item - 4] =
                    XK ? read_kmajor(base + xofs[item - 4] + s * 8192)
                       : *reinterpret_cast<const bf16x8_t*>(base + xbase + (item - 4) * 4096 + rofs[s]);
        };
        // the two MFMAs of slot i (0..7) of a quarter step on slice s
        auto mfma_pair = [&](int s, int i) {
            const int mt = i >> 1, n0 = (i & 1) * 2;
            acc[mt][n0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[s][mt], fx[s][n0], acc[mt][n0],
                                                                  0, 0, 0);
            acc[mt][n0 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[s][mt], fx[s][n0 + 1],
                                                                      acc[mt][n0 + 1], 0, 0, 0);
        };

        const int KT = K / kBlockK;
        // One 4-byte DMA per wavefront and k-step into a landing area nobody reads: it only pulls
        // the line into L2.  `warm` (see warm_row) must be a valid row pointer in every lane.
        // Not for two k-major operands (the weight-gradient products): measured there, the extra
        // L2 lookups cost as much as the early misses save.
        constexpr bool warming = !XK;
        unsigned char* const dump = smem + kStageBytes + w * 256;
        auto warm_step = [&](int kt) {
            // (with a Y that lacks k-rows of the last step, that step is not warmed: the lane's
            // line may be one of them)
            const int last = ytail && KT > 1 ? KT - 2 : KT - 1;
            const int kk = kt < last ? kt : last;
            dma_to_lds<4>(warm + kk * warm_stride, dump);
        };
        // Joins the wavefronts once this wavefront's DMA of the next stage has landed.  The warm-up
        // load issued after that DMA may still be in flight (loads complete in order).
        auto stage_barrier = [&](bool one_behind) {
            if (one_behind) asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        };
        if (warming)
            for (int p = 2; p < 2 + kWarmAhead; ++p) warm_step(p);
        issue_loads(0, 0);
        __syncthreads();                       // waits for the DMA (vmcnt) and joins the waves
        if (KT > 1) issue_loads(1, 1);
#pragma unroll
        for (int item = 0; item < 8; ++item) read_item(0, 0, item);
#pragma unroll
        for (int item = 0; item < 8; ++item) read_item(0, 1, item);

        // One k-step = four quarters of sixteen MFMAs, each quarter eight fenced slots of two MFMAs
        // plus the memory instructions that ride along, in this order:
        //   Q0  MFMA slice 0 | read slices 2 and 3 of this stage
        //   Q1  MFMA slice 1 |
        //   -- all of this stage has been read, the next stage has landed: workgroup barrier --
        //   Q2  MFMA slice 2 | DMA of step kt + 2, X half, into this stage | read slice 0 of kt + 1
        //   Q3  MFMA slice 3 | DMA of step kt + 2, Y half                  | read slice 1 of kt + 1
        // Every operand read is issued at least a quarter and a half before its first MFMA, so a
        // burst of DMA writes into LDS delays reads without draining the matrix pipe, and the DMA
        // issue is spread over half a step (left to the scheduler the sixteen DMA instructions
        // come out back to back and the matrix pipe idles behind their issue).
        // LOADS: step kt + 2 exists.  NEXT: step kt + 1 exists.  The tail steps skip the DMA so
        // that none is in flight when the workgroup ends.
        // BEHIND: the previous k-step issued a warm-up load after its DMA.
        auto kstep = [&](int kt, auto loads, auto next, bool behind) {
            constexpr bool LOADS = decltype(loads)::value, NEXT = decltype(next)::value;
            const int cur = kt & 1;
            unsigned char* const xs = smem + cur * kTileBytes + w * 8192;
            unsigned char* const ys = smem + 2 * kTileBytes + cur * kTileBytes + w * 8192;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_pair(0, i);
                read_item(cur, i < 4 ? 2 : 3, (2 * i) & 7);
                read_item(cur, i < 4 ? 2 : 3, (2 * i + 1) & 7);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_pair(1, i);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage_barrier(behind);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_pair(2, i);
                if (LOADS)
                    dma_to_lds<16>(xg[i] + (kt + 2) * xstep, xs + i * 1024);
                if (NEXT) read_item(cur ^ 1, 0, i);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_pair(3, i);
                if (LOADS)
                    dma_to_lds<16>(ysrc(i, kt + 2), ys + i * 1024);
                if (NEXT) read_item(cur ^ 1, 1, i);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (LOADS && warming) warm_step(kt + 2 + kWarmAhead);
        };
        // a step's barrier may leave one load in flight iff the step before it had LOADS and warmed
        int kt = 0;
        for (; kt + 2 < KT; ++kt) kstep(kt, std::true_type{}, std::true_type{}, warming && kt > 0);
        if (KT >= 2) {
            kstep(kt, std::false_type{}, std::true_type{}, warming && kt > 0);
            ++kt;
        }
        kstep(kt, std::false_type{}, std::false_type{}, false);
    }
};
typedef KMajorDirectT<true> KMajorCore;
typedef KMajorDirectT<false> MixedCore;

// ---------------------------------------------------------------------------------------------
// DirectCore: 4 wavefronts, global -> LDS DMA, aligned shapes only, both operands k-contiguous,
// v_mfma_f32_16x16x32_bf16
// ---------------------------------------------------------------------------------------------
// Against the same pipeline on the 32 x 32 x 16 form a plain product of the logits shape is 8 %
// faster (16-row operand reads, half the address arithmetic per k-step; with register-resident
// operands the two forms are level to 4 % apart).  It is the fastest of the cores, so products
// over a weight's row index are run on it against a copy of the weight transposed once per call.
struct DirectCore {
    static constexpr int kThreads = 256;
    static constexpr int kMT = 8;     // 16-wide c tiles per wavefront
    static constexpr int kNT = 8;     // 16-wide r tiles per wavefront
    static constexpr bool kCanGuard = false;
    typedef f32x4_t acc_t;
    static constexpr int kTile = 16, kRuns = 1, kGroups = 4;

    // acc[mt][nt][x]: r = nt * 16 + lane % 16, c = mt * 16 + 4 (lane / 16) + x inside the wavefront's
    // 128 x 128.
    struct Lane {
        int lane, grp, lrow, wr, wc;
        __device__ __forceinline__ Lane() {
            const int tid = threadIdx.x;
            lane = tid & 63;
            grp = lane >> 4;
            lrow = lane & 15;
            const int wave = tid >> 6;
            wr = wave & 1;
            wc = wave >> 1;
        }
        __device__ __forceinline__ int r(int nt) const { return wr * 128 + nt * 16 + lrow; }
        __device__ __forceinline__ int rbase(int nt) const { return wr * 128 + nt * 16; }
        __device__ __forceinline__ int cw(int mt, int /*q*/) const { return mt * 16 + grp * 4; }
        __device__ __forceinline__ int c(int mt, int q) const { return wc * kGroupC + cw(mt, q); }
    };

    // LDS row of a tile = 128 bytes = 8 chunks of 16 bytes; chunk kc of row `row` lives at slot
    // kc ^ ((row >> 1) & 7): sixteen consecutive rows at one kc then cover all 64 banks once.
    static __device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

    // The operands of one output block: D[r0 + r][c0 + c] = sum_k X[r0 + r][k] Y[c0 + c][k].
    // Requires K % 64 == 0, K >= 64, 16-byte aligned rows and r0 + 256 <= rows of X.
    // Y (without Y2) may end inside the block: it is read from its row rows_y - 1 in
    // place of the rows from rows_y on (the logits of a vocabulary that is not a multiple of the
    // block width), finite data of Y, and the caller discards those accumulator columns.
    // K_y (used with YTAIL, no Y2): if >= 0 and < K, the k extent Y has when X is zero-padded along k
    // beyond it (the logits of a hidden size that is not whole k-steps, X being the library's own
    // zero-padded copy of the hidden rows): the chunks of a row of Y beyond K_y are read from the
    // row's last chunk (K_y a multiple of 8) and meet zeros of X.
    // Y2: gated pair, see paired_row; rows_y is then the rows of Y and of Y2, the rows of the pair
    // beyond it are read from row 0 (finite data) and the caller discards those columns.
    // warm (see warm_row): the lane's warm-up row; warm_stride = elements between its line of one
    // k-step and the next.
    struct Block {
        const uint16_t* X;
        int64_t ldx;
        const uint16_t* Y;
        int64_t ldy;
        int rows_y, K, r0, c0;
        const uint16_t* warm;
        int64_t warm_stride;
        const uint16_t* Y2;
        int K_y;
    };

    // The k-loop's state: the DMA sources of the block whose operands are being fetched, the LDS
    // read offsets and the operand registers.  Used in two ways.
    //  * One block per workgroup: gemm() below.
    //  * A chain of blocks on one (persistent) workgroup: start(first); then for every block
    //    run(block, the block after it, acc) followed by the caller's epilogue; finish() after
    //    the last.  The last two k-steps of a block, which otherwise issue no DMA, fetch the
    //    first two k-steps of the block after it into the stages they free, so the next block's
    //    operands travel while the epilogue runs and no block but the first waits for a
    //    prologue.  The last block of a chain names itself as the block after it (the fetch is
    //    then wasted; finish() waits for it so that nothing is in flight when the workgroup
    //    ends).  Every block of a chain must have the same K, a multiple of 128 (the stages
    //    alternate: a block's step 0 must meet stage 0) and >= 256.  Between start() and
    //    finish() the first kLdsBytes of LDS belong to the chain: an epilogue that turns data
    //    around in LDS does it behind them.
    template <bool YTAIL>
    struct Pipe {
        unsigned char* smem;
        int w, lr, pc;                 // wavefront, the lane's row and chunk slot in a DMA instruction
        int rofs[2], xbase, ybase;     // LDS read offsets
        // the block the DMA works for: the lane's sources of k-step 0, its sources in the last
        // k-step where Y is shorter than K (clamped), the warm-up row
        const uint16_t* xg[8];
        const uint16_t* yg[8];
        const uint16_t* yg_tail[8];
        const uint16_t* warm;
        int64_t warm_stride;
        int KT_;
        bool ytail;
        // MFMA operands of the two k-slices of a step: fy[s][t], fx[s][t] for slice s
        bf16x8_t fy[2][8], fx[2][8];

        __device__ __forceinline__ explicit Pipe(unsigned char* smem_) : smem(smem_) {
            const int tid = threadIdx.x, lane = tid & 63;
            w = uniform(tid >> 6);
            const int wr = w & 1, wc = w >> 1;
            const int l15 = lane & 15, g = lane >> 4;
            // One DMA instruction moves 8 rows x 128 bytes: lane -> (row = lane / 8, LDS chunk slot
            // = lane % 8); the lane fetches the global chunk that belongs in its slot.  Wave w owns
            // rows [64 w, 64 w + 64) of both operand tiles: 8 instructions per operand per k-step.
            lr = lane >> 3;
            pc = lane & 7;
            // Operand reads.  A k-step is two slices of 32 k; lane (row l15 of a 16-row tile,
            // k-group g) reads the 16-byte chunk 4 s + g of its row: one read per operand.
#pragma unroll
            for (int s = 0; s < 2; ++s) rofs[s] = ((4 * s + g) ^ swz(l15)) * 16;
            xbase = (wr * 128 + l15) * 128;
            ybase = 2 * kTileBytes + (wc * kGroupC + l15) * 128;
        }
        __device__ __forceinline__ void target(const Block& b) {
            KT_ = b.K / kBlockK;
            ytail = YTAIL && b.K_y >= 0 && b.K_y < b.K;
            warm = b.warm;
            warm_stride = b.warm_stride;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int row = (w * 8 + q) * 8 + lr;
                const int kc = pc ^ swz(row);
                xg[q] = b.X + (int64_t)(b.r0 + row) * b.ldx + kc * 8;
                if (b.Y2) {                         // gated pair
                    bool valid;
                    yg[q] = paired_row(b.Y, b.Y2, b.ldy, b.c0, row, b.rows_y, valid) + kc * 8;   // (missing rows: row 0)
                } else {
                    const int yrow = b.c0 + row < b.rows_y ? b.c0 + row : b.rows_y - 1;    // (the clamp: see Block)
                    yg[q] = b.Y + (int64_t)yrow * b.ldy + kc * 8;
                    if (YTAIL) {
                        const int k = (KT_ - 1) * kBlockK + kc * 8;
                        yg_tail[q] = b.Y + (int64_t)yrow * b.ldy + (ytail && k >= b.K_y ? b.K_y - 8 : k);
                    }
                }
            }
        }
        __device__ __forceinline__ const uint16_t* ysrc(int q, int kt) const {
            if (YTAIL) return (ytail && kt == KT_ - 1) ? yg_tail[q] : yg[q] + kt * kBlockK;
            return yg[q] + kt * kBlockK;
        }
        __device__ __forceinline__ void issue_loads(int stage, int kt) {
            unsigned char* xs = smem + stage * kTileBytes + w * 8192;
            unsigned char* ys = smem + 2 * kTileBytes + stage * kTileBytes + w * 8192;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                dma_to_lds<16>(xg[q] + kt * kBlockK, xs + q * 1024);
                dma_to_lds<16>(ysrc(q, kt), ys + q * 1024);
            }
        }
        // item 0..7: the Y operand of accumulator row t = item, 8..15: the X operand of column t
        __device__ __forceinline__ void read_item(int stage, int s, int item) {
            const unsigned char* base = smem + stage * kTileBytes + rofs[s];
            if (item < 8) fy[s][item] = *reinterpret_cast<const bf16x8_t*>(base + ybase + item * 2048);
            else fx[s][item - 8] = *reinterpret_cast<const bf16x8_t*>(base + xbase + (item - 8) * 2048);
        }
        // the four MFMAs of slot i (0..15) of a slice
        __device__ __forceinline__ void mfma_quad(acc_t (&acc)[kMT][kNT], int s, int i) {
            const int mt = i >> 1, n0 = (i & 1) * 4;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                acc[mt][n0 + d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fy[s][mt], fx[s][n0 + d],
                                                                          acc[mt][n0 + d], 0, 0, 0);
        }
        // One 4-byte DMA per wavefront and k-step into a landing area nobody reads: it only pulls
        // the line into L2.  `warm` must be a valid row pointer in every lane.  Steps beyond the
        // targeted block's last are steps of `ahead`, the block after it in a chain (or clamped).
        __device__ __forceinline__ void warm_step(int kt, const Block* ahead) {
            unsigned char* const dump = smem + kStageBytes + w * 256;
            if (ahead != nullptr && kt >= KT_) {
                // (the next block's first steps: whole k-steps of Y, K >= 256)
                dma_to_lds<4>(ahead->warm + (kt - KT_) * ahead->warm_stride, dump);
                return;
            }
            // (with a Y that lacks k of the last step, that step is not warmed: the lane's line
            // may lie beyond K_y)
            const int last = ytail && KT_ > 1 ? KT_ - 2 : KT_ - 1;
            const int kk = kt < last ? kt : last;
            dma_to_lds<4>(warm + kk * warm_stride, dump);
        }
        // Joins the wavefronts once this wavefront's DMA of the next stage has landed.  The warm-up
        // load issued after that DMA may still be in flight (loads complete in order).
        static __device__ __forceinline__ void stage_barrier(bool one_behind) {
            if (one_behind) asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }

        // One k-step = two slices of 64 MFMAs, each slice sixteen fenced slots of four MFMAs (64
        // cycles) plus the memory instructions that ride along, in this order:
        //   slice 0, slots 0..7    | read slice 1 of this stage (two operands per slot)
        //   slice 0, slots 8..15   |
        //   -- all of this stage has been read, the next stage has landed: workgroup barrier --
        //   slice 1, slots 0..7    | DMA of step kt + 2, X half, into this stage | read slice 0 of kt + 1
        //   slice 1, slots 8..15   | DMA of step kt + 2, Y half                  | read slice 0 of kt + 1
        // Every operand read is issued at least half a slice before its first MFMA, so a burst of
        // DMA writes into LDS delays reads without draining the matrix pipe, and the DMA issue is
        // spread over half a step (left to the scheduler the sixteen DMA instructions come out
        // back to back and the matrix pipe idles behind their issue).  Inside a slot the MFMAs
        // go first (the sched_group_barrier calls): the wait the compiler puts before a slot's
        // first MFMA then covers reads issued long ago, not the slot's own (1.5 % of the kernel).
        // kt: the step computed (its stage is kt & 1).  LOADS: the DMA of step dkt + 2 of the
        // targeted block is issued (dkt = kt, or kt - KT when the target is the next block of a
        // chain).  NEXT: step kt + 1 exists.  Steps without LOADS leave no DMA in flight.
        // BEHIND: the previous k-step issued a warm-up load after its DMA.
        template <bool LOADS, bool NEXT>
        __device__ __forceinline__ void kstep(acc_t (&acc)[kMT][kNT], int kt, int dkt, bool behind,
                                              const Block* ahead) {
            const int cur_stage = kt & 1;
            unsigned char* const xs = smem + cur_stage * kTileBytes + w * 8192;
            unsigned char* const ys = smem + 2 * kTileBytes + cur_stage * kTileBytes + w * 8192;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_quad(acc, 0, i);
                read_item(cur_stage, 1, 2 * i);
                read_item(cur_stage, 1, 2 * i + 1);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 8; i < 16; ++i) {
                mfma_quad(acc, 0, i);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage_barrier(behind);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                mfma_quad(acc, 1, i);
                if (LOADS) dma_to_lds<16>(xg[i] + (dkt + 2) * kBlockK, xs + i * 1024);
                if (NEXT) read_item(cur_stage ^ 1, 0, i);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                if (LOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (NEXT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 8; i < 16; ++i) {
                mfma_quad(acc, 1, i);
                if (LOADS) dma_to_lds<16>(ysrc(i - 8, dkt + 2), ys + (i - 8) * 1024);
                if (NEXT) read_item(cur_stage ^ 1, 0, i);
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                if (LOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (NEXT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (LOADS) warm_step(dkt + 2 + kWarmAhead, ahead);
        }

        // ---- one block per workgroup
        __device__ __forceinline__ void single(const Block& b, acc_t (&acc)[kMT][kNT]) {
            const int KT = b.K / kBlockK;
            target(b);
            for (int p = 2; p < 2 + kWarmAhead; ++p) warm_step(p, nullptr);
            issue_loads(0, 0);
            __syncthreads();                   // waits for the DMA (vmcnt) and joins the waves
            if (KT > 1) issue_loads(1, 1);
#pragma unroll
            for (int item = 0; item < 16; ++item) read_item(0, 0, item);
            // a step's barrier may leave one load in flight iff the step before it had LOADS and warmed
            int kt = 0;
            for (; kt + 2 < KT; ++kt) kstep<true, true>(acc, kt, kt, kt > 0, nullptr);
            if (KT >= 2) {
                kstep<false, true>(acc, kt, kt, kt > 0, nullptr);
                ++kt;
            }
            kstep<false, false>(acc, kt, kt, false, nullptr);
        }

        // ---- a chain of blocks
        __device__ __forceinline__ void start(const Block& first) {
            target(first);
            for (int p = 2; p < 2 + kWarmAhead; ++p) warm_step(p, nullptr);
            issue_loads(0, 0);
            issue_loads(1, 1);
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");     // step 0 has landed (loads complete in order)
        }
        // acc += the product of `cur`, the targeted block, whose k-step 0 this wavefront's DMA has
        // landed and whose k-step 1 is in flight; fetches the first two k-steps of `next`, targets
        // it and returns when this wavefront's part of its k-step 0 has landed.  The stores of the
        // caller's epilogue are never waited for on their own: the barrier of the next block's
        // k-step 0, half a step in, covers them together with the DMA of its k-step 1.
        __device__ __forceinline__ void run(const Block& cur, const Block& next, acc_t (&acc)[kMT][kNT]) {
            const int KT = uniform(cur.K / kBlockK);
            // every wavefront's part of k-step 0 has landed, and all are done with the block before
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
            for (int item = 0; item < 16; ++item) read_item(0, 0, item);
            int kt = 0;
            for (; kt + 2 + kWarmAhead < KT; ++kt) kstep<true, true>(acc, kt, kt, kt > 0, nullptr);
            // (the warm-up loads of these steps are for the first steps of `next`)
            for (; kt + 2 < KT; ++kt) kstep<true, true>(acc, kt, kt, kt > 0, &next);
            target(next);
            kstep<true, true>(acc, kt, -2, true, nullptr);
            kstep<true, false>(acc, kt + 1, -1, true, nullptr);
            // all but the 16 DMA instructions of the last half step and the warm-up load behind them
            asm volatile("s_waitcnt vmcnt(17)" ::: "memory");
        }
        __device__ __forceinline__ void finish() { stage_barrier(false); }
    };

    // One block on its own.  GUARD must be false.
    template <bool GUARD, bool YTAIL = false>
    static __device__ __forceinline__ void gemm(const uint16_t* __restrict__ X, int64_t ldx,
                                                int /*rows_x*/, const uint16_t* __restrict__ Y,
                                                int64_t ldy, int rows_y, int K, int r0, int c0,
                                                unsigned char* smem, acc_t (&acc)[kMT][kNT],
                                                const uint16_t* warm, int64_t warm_stride = kBlockK,
                                                const uint16_t* Y2 = nullptr, int K_y = -1) {
        static_assert(!GUARD, "the DMA cores have no bounds checks");
        const Block b = {X, ldx, Y, ldy, rows_y, K, r0, c0, warm, warm_stride, Y2, K_y};
        Pipe<YTAIL> pipe(smem);
        pipe.single(b, acc);
    }
};

// ---------------------------------------------------------------------------------------------
// out[c][r] = in[r][c] (bf16), zeros for rows <= r < the 64 rows of the last piece
// ---------------------------------------------------------------------------------------------
// Weights that a product contracts over their row index are transposed once per call, so that
// the product reads both operands along their rows (DirectCore).  in: [rows, ld_in], cols a
// multiple of 8, 16-byte aligned rows; out: [cols, ld_out], ld_out >= rows rounded up to 64.  One
// workgroup of 256 turns a 64 x 64 piece around in LDS; grid = (ceil(rows / 64), ceil(cols / 64)).
static __global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ in, int rows,
                                                                    int cols, int64_t ld_in,
                                                                    uint16_t* __restrict__ out, int64_t ld_out) {
    __shared__ uint16_t piece[64][64 + 2];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int t = threadIdx.x;
    // in: 64 rows x 8 chunks of 8 columns; thread -> (row t / 8 + 32 j, chunk t % 8)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = t / 8 + 32 * j, cc = (t % 8) * 8;
        u32x4_t x = {0u, 0u, 0u, 0u};
        if (r0 + r < rows && c0 + cc < cols)
            x = *reinterpret_cast<const u32x4_t*>(in + (int64_t)(r0 + r) * ld_in + c0 + cc);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            piece[r][cc + 2 * q] = (uint16_t)(x[q] & 0xffffu);
            piece[r][cc + 2 * q + 1] = (uint16_t)(x[q] >> 16);
        }
    }
    __syncthreads();
    // out: 64 rows (columns of in) x 8 chunks of 8
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int c = t / 8 + 32 * j, rc = (t % 8) * 8;
        if (c0 + c >= cols) continue;
        u32x4_t y;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            y[q] = (uint32_t)piece[rc + 2 * q][c] | ((uint32_t)piece[rc + 2 * q + 1][c] << 16);
        *reinterpret_cast<u32x4_t*>(out + (int64_t)(c0 + c) * ld_out + r0 + rc) = y;
    }
}

// ---------------------------------------------------------------------------------------------
// Epilogues shared by the kernels built on the cores (written against the cores' layout traits)
// ---------------------------------------------------------------------------------------------
constexpr int kTurnPitch = 272;     // bytes per row of the LDS turn-around area: 256 + 16 of padding
// LDS of a kernel whose workgroups run chains of blocks on DirectCore (gemm_chain): the epilogue's
// turn-around area (4 wavefronts x 16 rows) lies behind the stages and the warm-up landing area,
// which belong to the next block's DMA while the epilogue runs.
constexpr int kChainTurnOffset = kLdsBytes;
constexpr int kChainLdsBytes = kChainTurnOffset + 4 * 16 * kTurnPitch;

template <class Core>
__device__ __forceinline__ void zero_acc(typename Core::acc_t (&acc)[Core::kMT][Core::kNT]) {
#pragma unroll
    for (int mt = 0; mt < Core::kMT; ++mt)
#pragma unroll
        for (int nt = 0; nt < Core::kNT; ++nt)
#pragma unroll
            for (int j = 0; j < 4 * Core::kRuns; ++j) acc[mt][nt][j] = 0.f;
}

// D[(r0 + r) * ldd + c0 + c] = bf16(acc) for the block's 256 x 256 accumulators, D row-major with c
// contiguous.  In the accumulators a lane holds 4 consecutive c of one r, so a direct store would
// scatter 8-byte pieces over many rows per instruction: each wavefront instead turns its
// kTile x 128 pieces around in LDS (free once the k-loop is over; each wavefront has its own region
// and LDS serves a wavefront's accesses in order, so no barrier is needed) and stores whole
// 256-byte row segments (non-temporal stores: the output is a stream that nothing reads back while
// it is in L2, and it would push operand lines out of there; -1 % on the K = 4096 products).
// `smem`: 4 * kTile * kTurnPitch bytes of LDS for this.
// GUARD: rows >= rows_out and 8-column chunks beyond cols_out are not written.
template <class Core, bool GUARD>
__device__ __forceinline__ void store_block_bf16(const typename Core::acc_t (&acc)[Core::kMT][Core::kNT],
                                                 uint16_t* __restrict__ D, int64_t ldd, int r0,
                                                 int c0, int rows_out, int cols_out,
                                                 unsigned char* smem) {
    const typename Core::Lane lp;
    unsigned char* const tw = smem + (threadIdx.x >> 6) * (Core::kTile * kTurnPitch);
    const int lrow = lp.lane >> 4, lcol = lp.lane & 15;            // 4 rows x 16 chunks of 16 B
    const int gc = c0 + lp.wc * kGroupC + lcol * 8;
#pragma unroll
    for (int nt = 0; nt < Core::kNT; ++nt) {
#pragma unroll
        for (int mt = 0; mt < Core::kMT; ++mt)
#pragma unroll
            for (int q = 0; q < Core::kRuns; ++q) {
                bf16x4_t o;
#pragma unroll
                for (int x = 0; x < 4; ++x) o[x] = (__bf16)acc[mt][nt][q * 4 + x];
                *reinterpret_cast<bf16x4_t*>(tw + lp.lrow * kTurnPitch + lp.cw(mt, q) * 2) = o;
            }
#pragma unroll
        for (int it = 0; it < Core::kTile / 4; ++it) {
            const int row = it * 4 + lrow;
            const int gr = r0 + lp.rbase(nt) + row;
            const u32x4_t v = *reinterpret_cast<const u32x4_t*>(tw + row * kTurnPitch + lcol * 16);
            if (!GUARD || (gr < rows_out && gc + 8 <= cols_out))
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(D + (int64_t)gr * ldd + gc));
        }
    }
}

// out[(c0 + c) * ld + r0 + r] (+)= acc: the transposed fp32 accumulate used by the weight-gradient
// GEMMs.  r runs along the MFMA lane dimension, so each accumulator register of a wavefront
// covers runs of kTile consecutive floats of rows of `out` and the accumulate is one
// fire-and-forget fp32 atomic add per register (a plain store when `first`).  Each element
// belongs to exactly one lane per launch; launches on one stream are ordered, so the sums are
// formed in launch order: deterministic.  Rows r >= r_valid and c >= c_valid are skipped.
template <class Core, bool GUARD>
__device__ __forceinline__ void accumulate_block_f32(const typename Core::acc_t (&acc)[Core::kMT][Core::kNT],
                                                     float* __restrict__ out, int64_t ld, int r0,
                                                     int c0, int r_valid, int c_valid, bool first) {
    const typename Core::Lane lp;
#pragma unroll
    for (int nt = 0; nt < Core::kNT; ++nt) {
        const int r = r0 + lp.r(nt);
        if (r >= r_valid) continue;
#pragma unroll
        for (int mt = 0; mt < Core::kMT; ++mt)
#pragma unroll
            for (int j = 0; j < 4 * Core::kRuns; ++j) {
                const int c = c0 + lp.c(mt, j >> 2) + (j & 3);
                if (c >= c_valid) continue;
                float* dst = out + (int64_t)c * ld + r;
                if (first) *dst = acc[mt][nt][j];
                else unsafeAtomicAdd(dst, acc[mt][nt][j]);
            }
    }
}

}  // namespace alst
