// Sequence-tiled gated MLP and sequence-tiled linear layer for gfx950: kernels and the C ABI
// (alst_mlp.h, alst_linear.h).
//
// Paper, subsection "TiledMLP": forward and backward of the MLP are run on tiles of the sequence,
// the [tile, intermediate] activations exist only for the tile in flight and backward recomputes
// them.  Per tile of T rows, all contractions on the block GEMM of gemm_tile.h (operands with the
// contraction index contiguous):
//
//   forward    a  = silu(x Wg^T) * (x Wu^T)   gated_kernel: both products in one block, SwiGLU in
//                                             the epilogue, g and u never reach memory
//              y  = a Wd^T
//   backward   da = dy Wd                     against Wd^T, transposed once per call
//              a, [dg | du]                   gated_kernel again (g and u recomputed), its epilogue
//                                             reads da; written into the rows of the tile's group
//              dx = dg Wg + du Wu             one contraction over the 2 I columns of [dg | du]
//                                             against [Wg | Wu]^T, transposed once per call
//                                             (H or I not a multiple of 64: the weights as they are,
//                                             k-major operands, dx as two contractions over I)
//   per group  dWg += dg^T x, dWu += du^T x, dWd += dy^T a   (fp32, contraction over the group's rows)
//
// As in the cross-entropy path the weight gradients are accumulated once per group of tiles
// (about 16384 rows), so the read-modify-write of the fp32 sums is paid once per group.  Their
// operands have the contraction index (the token row) as the slow index and are read as they are
// by the k-major cores: x and dy straight from the caller's arrays, a and [dg | du] from the
// group's buffers.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <mutex>
#include <stdint.h>
#include <math.h>

#include "../../include/alst_mlp.h"
#include "../../include/alst_linear.h"
#include "gemm_tile.h"
#include "common.h"

namespace alst {

constexpr int kMlpGroupRows = 16384;
constexpr int kMlpGroupMax = 8;

struct MlpLayout {
    int64_t Tp, Kg;        // tile rows rounded up to 256; rows a weight-gradient group can hold
    int g;                 // tiles per weight-gradient group
    size_t a, da, dgu, wdt, wgut, acc_g, acc_u, acc_d, total;
    bool weights_t;        // backward multiplies by transposed copies of the weights
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static MlpLayout make_mlp_layout(int64_t N, int64_t H, int64_t I, int64_t tile, bool backward,
                                 uint32_t flags) {
    MlpLayout L = {};
    const int64_t T = tile < N ? tile : N;
    L.Tp = (T + 255) / 256 * 256;
    int64_t g = kMlpGroupRows / L.Tp;
    L.g = (int)(g < 1 ? 1 : (g > kMlpGroupMax ? kMlpGroupMax : g));
    L.Kg = (int64_t)L.g * L.Tp;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    // backward keeps a and [dg | du] of the whole group, each tile behind the one before
    L.a = take((size_t)(backward ? L.Kg : L.Tp) * I * 2);
    if (backward) {
        L.da = take((size_t)L.Tp * I * 2);
        L.dgu = take((size_t)L.Kg * 2 * I * 2);
        // Wd transposed [I, H] and [Wg | Wu] transposed [H, 2 I], made once per call: da = dy Wd and
        // dx = [dg | du] [Wg ; Wu] then read both operands along their rows (the fastest layout
        // of the block GEMM).  For H and I that are whole k-steps; else the weights are read as
        // they are.
        L.weights_t = H % kBlockK == 0 && I % kBlockK == 0;
        L.wdt = take(L.weights_t ? (size_t)I * H * 2 : 0);
        L.wgut = take(L.weights_t ? (size_t)H * 2 * I * 2 : 0);
        // fp32 overwrite outputs hold the sums themselves
        const bool in_out = (flags & ALST_FLAG_DW_FP32) && !(flags & ALST_FLAG_DW_ACCUMULATE);
        L.acc_g = take(in_out ? 0 : (size_t)I * H * 4);
        L.acc_u = take(in_out ? 0 : (size_t)I * H * 4);
        L.acc_d = take(in_out ? 0 : (size_t)H * I * 4);
    }
    L.total = o;
    return L;
}

// ---------------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------------
struct LinearParams {
    const uint16_t* X;       // [rows_x, ldx]   k contiguous
    const uint16_t* Y;       // [rows_y, ldy]   k contiguous: D[r][c] = sum_k X[r][k] Y[c][k], bf16
                             // [K, ldy]        k-major (y_kmajor; a weight matrix contracted over its
                             //                 row index, as it is): D[r][c] = sum_k X[r][k] Y[k][c],
                             //                 rows_y = its number of columns
    uint16_t* D;             // [.., ldd]
    const uint16_t* X2;      // second product summed into the same D (y_kmajor only, same K and
    const uint16_t* Y2;      // leading dimensions), or null
    int64_t ldx, ldy, ldd;
    int rows_x, rows_y, K;
    int rows_out, cols_out;  // guarded builds write only r < rows_out, 8-column chunks below cols_out
    int y_kmajor;
};

// Up to three independent products in one launch: their patches of output blocks are numbered
// through (gemm_tile.h), so the XCDs stay evenly loaded and the tail of one product is filled by
// the first workgroups of the next instead of leaving compute units idle.
constexpr int kMaxBatch = 3;
struct BatchMap {
    PatchGrid g[kMaxBatch];
    int first_patch[kMaxBatch + 1];      // first_patch[i] .. first_patch[i + 1]: patches of part i
    int n;
    // which part and which of its blocks a workgroup works on; false for padding workgroups
    __device__ __forceinline__ bool locate(int bid, int& which, int& tr, int& tc, int& PR, int& PC) const {
        int P, w;
        patch_of_block(bid, P, w);
        if (P >= first_patch[n]) return false;
        which = 0;
#pragma unroll
        for (int i = 1; i < kMaxBatch; ++i)
            if (i < n && P >= first_patch[i]) which = i;
        PR = g[which].PR;
        PC = g[which].PC;
        return tile_in_patch(g[which], P - first_patch[which], w, tr, tc);
    }
};
struct LinearBatch {
    LinearParams p[kMaxBatch];
    BatchMap map;
};

template <class Core, bool GUARD>
__global__ __launch_bounds__(Core::kThreads) void linear_kernel(const LinearBatch b) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    extern __shared__ __align__(16) unsigned char smem[];
    int which, tr, tc, PR, PC;
    if (!b.map.locate(blockIdx.x, which, tr, tc, PR, PC)) return;
    const LinearParams& p = b.p[which];
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    constexpr bool kMixed = std::is_same<Core, MixedCore>::value || std::is_same<Core, StagedMixedCore>::value;
    if constexpr (kMixed) {
        int64_t step = 0;
        const uint16_t* warm = Core::kCanGuard ? nullptr
                                               : warm_line_mixed(PR, PC, p.X, p.ldx, r0, tr, p.Y, p.ldy,
                                                                 c0, tc, step);
        Core::template gemm<GUARD>(p.X, p.ldx, p.rows_x, p.Y, p.ldy, p.rows_y, p.K, r0, c0, smem, acc, warm,
                                   step);
        if (p.X2) {
            __syncthreads();        // every wavefront is done with the first product's LDS stages
            warm = Core::kCanGuard ? nullptr
                                   : warm_line_mixed(PR, PC, p.X2, p.ldx, r0, tr, p.Y2, p.ldy, c0, tc, step);
            Core::template gemm<GUARD>(p.X2, p.ldx, p.rows_x, p.Y2, p.ldy, p.rows_y, p.K, r0, c0, smem, acc,
                                       warm, step);
        }
    } else {
        const uint16_t* warm = Core::kCanGuard ? nullptr
                                               : warm_row(PR, PC, p.X, p.ldx, r0, tr, p.Y, p.ldy, c0, tc);
        Core::template gemm<GUARD>(p.X, p.ldx, p.rows_x, p.Y, p.ldy, p.rows_y, p.K, r0, c0, smem, acc, warm);
    }
    store_block_bf16<Core, GUARD>(acc, p.D, p.ldd, r0, c0, p.rows_out, p.cols_out, smem);
}

// The k-contiguous products on persistent workgroups: one workgroup per compute unit walks the
// launch's blocks bid = blockIdx.x, blockIdx.x + gridDim.x, ... (the same block numbering as
// linear_kernel, so the 32 workgroups of an XCD still share a patch) and fetches the first two
// k-steps of its next block while the current block's last two k-steps and epilogue run
// (DirectCore::Pipe).  total = the launch's block numbers (grid_for_patches).  Every product of
// the launch has the same K, a multiple of 128 and >= 256.
__global__ __launch_bounds__(DirectCore::kThreads) void linear_chain_kernel(const LinearBatch b, int total) {
    typedef DirectCore Core;
    extern __shared__ __align__(16) unsigned char smem[];
    // the next block number from `bid` on that is not padding, or -1
    auto next_block = [&](int bid, Core::Block& blk, int& which) {
        for (; bid < total; bid += gridDim.x) {
            int tr, tc, PR, PC;
            if (!b.map.locate(bid, which, tr, tc, PR, PC)) continue;
            const LinearParams& p = b.p[which];
            const int r0 = tr * kBlockR, c0 = tc * kBlockC;
            blk = {uniform(p.X), uniform(p.ldx), uniform(p.Y), uniform(p.ldy), uniform(p.rows_y), uniform(p.K),
                   uniform(r0), uniform(c0), warm_row(PR, PC, p.X, p.ldx, r0, tr, p.Y, p.ldy, c0, tc), kBlockK,
                   nullptr, -1};
            which = uniform(which);
            return uniform(bid);
        }
        return -1;
    };
    Core::Block cur, nxt;
    int which, which_next = 0;
    int bid = next_block(blockIdx.x, cur, which);
    if (bid < 0) return;
    Core::Pipe<false> pipe(smem);
    pipe.start(cur);
    while (bid >= 0) {
        const int nbid = next_block(bid + gridDim.x, nxt, which_next);
        if (nbid < 0) {            // the last block: the chain's fetch goes to this block again, unused
            nxt = cur;
            which_next = which;
        }
        typename Core::acc_t acc[Core::kMT][Core::kNT];
        zero_acc<Core>(acc);
        pipe.run(cur, nxt, acc);
        const LinearParams& p = b.p[which];
        store_block_bf16<Core, false>(acc, p.D, p.ldd, cur.r0, cur.c0, p.rows_out, p.cols_out,
                                      smem + kChainTurnOffset);
        cur = nxt;
        which = which_next;
        bid = nbid;
    }
    pipe.finish();
}

// Gate and up projections of a tile with the SwiGLU in the epilogue: the block's Y rows are the
// gated pair (Wg, Wu) of gemm_tile.h, so every lane holds g and u of the same elements and neither
// reaches memory.
//   forward   a = silu(g) * u
//   backward  also reads da and writes dg = da * u * silu'(g), du = da * silu(g) as [dg | du]
// g and u enter the SwiGLU as the fp32 accumulators.
struct GatedParams {
    const uint16_t* X;       // [rows_x, ldx]   the tile's rows of x
    const uint16_t* Wg;      // [I, ldw]
    const uint16_t* Wu;      // [I, ldw]
    const uint16_t* da;      // [rows_out, I]   backward
    uint16_t* a;             // [rows_out, I]
    uint16_t* dgu;           // [rows_out, 2I]  backward
    int64_t ldx, ldw;
    int rows_x, I, K;
    int rows_out;            // rows written; those from rows_x on come out as zeros
    PatchGrid grid;
};

// The SwiGLU epilogue of a block whose accumulators hold g (tiles mt < kMT / 2) and u (tile mt + kMT / 2)
// of the same elements.  CHECK: rows >= rows_out and 8-column chunks beyond I are neither read nor
// written.  tw: this wavefront's LDS turn-around region (kTile rows of kTurnPitch bytes).
template <class Core, bool BWD, bool CHECK>
__device__ __forceinline__ void gated_epilogue(const GatedParams& p,
                                               const typename Core::acc_t (&acc)[Core::kMT][Core::kNT],
                                               int r0, int c0, unsigned char* tw) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    constexpr int kHalfMT = kMT / 2;
    constexpr bool kCheckCols = CHECK;
    // Per wavefront and accumulator column nt: kTile rows x 64 columns of I.  Everything that goes
    // to or comes from memory is turned around in the wavefront's own LDS region (as in
    // store_block_bf16) so that global accesses are whole 128-byte row segments.
    const typename Core::Lane lp;
    constexpr int kRuns = Core::kRuns, kTile = Core::kTile;
    const int lrow = lp.lane >> 3, lcol = lp.lane & 7;             // 8 rows x 8 chunks of 16 B
    const int gc = (c0 >> 1) + lp.wc * 64 + lcol * 8;              // this lane's 8 columns of I
    const bool col_ok = !kCheckCols || gc + 8 <= p.I;
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) {
        const int row0 = r0 + lp.rbase(nt);
        // the lane's own elements: row lrow of the tile, columns cw(mt, q) + x of the wavefront's 64
        auto own = [&](int mt, int q) { return tw + lp.lrow * kTurnPitch + lp.cw(mt, q) * 2; };
        auto store_rows = [&](const bf16x4_t (&v)[kHalfMT][kRuns], uint16_t* dst, int64_t ld) {
#pragma unroll
            for (int mt = 0; mt < kHalfMT; ++mt)
#pragma unroll
                for (int q = 0; q < kRuns; ++q) *reinterpret_cast<bf16x4_t*>(own(mt, q)) = v[mt][q];
#pragma unroll
            for (int it = 0; it < kTile / 8; ++it) {
                const int row = it * 8 + lrow;
                const u32x4_t val = *reinterpret_cast<const u32x4_t*>(tw + row * kTurnPitch + lcol * 16);
                if (!kCheckCols || (row0 + row < p.rows_out && col_ok))
                    *reinterpret_cast<u32x4_t*>(dst + (int64_t)(row0 + row) * ld + gc) = val;
            }
        };
        bf16x4_t d[kHalfMT][kRuns];
        if (BWD) {
#pragma unroll
            for (int it = 0; it < kTile / 8; ++it) {
                const int row = it * 8 + lrow;
                const bool ok = !kCheckCols || (row0 + row < p.rows_out && col_ok);
                const u32x4_t val = ok ? *reinterpret_cast<const u32x4_t*>(p.da + (int64_t)(row0 + row) * p.I + gc)
                                       : zero4;
                *reinterpret_cast<u32x4_t*>(tw + row * kTurnPitch + lcol * 16) = val;
            }
#pragma unroll
            for (int mt = 0; mt < kHalfMT; ++mt)
#pragma unroll
                for (int q = 0; q < kRuns; ++q) d[mt][q] = *reinterpret_cast<const bf16x4_t*>(own(mt, q));
        }
        bf16x4_t oa[kHalfMT][kRuns], og[kHalfMT][kRuns], ou[kHalfMT][kRuns];
#pragma unroll
        for (int mt = 0; mt < kHalfMT; ++mt)
#pragma unroll
            for (int q = 0; q < kRuns; ++q)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float g = acc[mt][nt][q * 4 + x], u = acc[mt + kHalfMT][nt][q * 4 + x];
                    const float sg = 1.f / (1.f + __expf(-g));
                    const float silu = g * sg;
                    oa[mt][q][x] = (__bf16)(silu * u);
                    if (BWD) {
                        const float dd = (float)d[mt][q][x];
                        og[mt][q][x] = (__bf16)(dd * u * (sg * (1.f + g * (1.f - sg))));
                        ou[mt][q][x] = (__bf16)(dd * silu);
                    }
                }
        store_rows(oa, p.a, p.I);
        if (BWD) {
            store_rows(og, p.dgu, 2 * (int64_t)p.I);
            store_rows(ou, p.dgu + p.I, 2 * (int64_t)p.I);
        }
    }
}

// CGUARD: I ends inside the block's 128 columns (the unguarded core reads row 0 of Wg / Wu in place
// of the missing rows; the epilogue skips those columns).
template <class Core, bool GUARD, bool BWD, bool CGUARD = false>
__global__ __launch_bounds__(Core::kThreads) void gated_kernel(const GatedParams p) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    static_assert(kMT * Core::kTile == kGroupC, "a wavefront's 128 Y rows: 64 of Wg, then the same 64 of Wu");
    extern __shared__ __align__(16) unsigned char smem[];
    int P, w, tr, tc;
    patch_of_block(blockIdx.x, P, w);
    if (P >= p.grid.patches() || !tile_in_patch(p.grid, P, w, tr, tc)) return;
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;      // c0 / 2 = first of the block's 128 columns of I

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    const uint16_t* warm = Core::kCanGuard ? nullptr
                                           : warm_row(p.grid.PR, p.grid.PC, p.X, p.ldx, r0, tr, p.Wg,
                                                      p.ldw, c0, tc, p.Wu, p.I);
    Core::template gemm<GUARD>(p.X, p.ldx, p.rows_x, p.Wg, p.ldw, p.I, p.K, r0, c0, smem, acc, warm,
                               kBlockK, p.Wu);
    gated_epilogue<Core, BWD, GUARD || CGUARD>(p, acc, r0, c0, smem + (threadIdx.x >> 6) * (32 * kTurnPitch));
}

// The same on persistent workgroups of the unguarded core (see linear_chain_kernel): K = H a
// multiple of 128 and >= 256.  total = the launch's block numbers.
template <bool BWD, bool CGUARD>
__global__ __launch_bounds__(DirectCore::kThreads) void gated_chain_kernel(const GatedParams p, int total) {
    typedef DirectCore Core;
    extern __shared__ __align__(16) unsigned char smem[];
    auto next_block = [&](int bid, Core::Block& blk) {
        for (; bid < total; bid += gridDim.x) {
            int P, w, tr, tc;
            patch_of_block(bid, P, w);
            if (P >= p.grid.patches() || !tile_in_patch(p.grid, P, w, tr, tc)) continue;
            const int r0 = tr * kBlockR, c0 = tc * kBlockC;
            blk = {uniform(p.X), p.ldx, uniform(p.Wg), p.ldw, p.I, p.K, uniform(r0), uniform(c0),
                   warm_row(p.grid.PR, p.grid.PC, p.X, p.ldx, r0, tr, p.Wg, p.ldw, c0, tc, p.Wu, p.I), kBlockK,
                   uniform(p.Wu), -1};
            return uniform(bid);
        }
        return -1;
    };
    Core::Block cur, nxt;
    int bid = next_block(blockIdx.x, cur);
    if (bid < 0) return;
    Core::Pipe<false> pipe(smem);
    pipe.start(cur);
    unsigned char* const tw = smem + kChainTurnOffset + (threadIdx.x >> 6) * (Core::kTile * kTurnPitch);
    while (bid >= 0) {
        const int nbid = next_block(bid + gridDim.x, nxt);
        if (nbid < 0) nxt = cur;        // the last block: the chain's fetch goes to this block again, unused
        typename Core::acc_t acc[Core::kMT][Core::kNT];
        zero_acc<Core>(acc);
        pipe.run(cur, nxt, acc);
        gated_epilogue<Core, BWD, CGUARD>(p, acc, cur.r0, cur.c0, tw);
        cur = nxt;
        bid = nbid;
    }
    pipe.finish();
}

struct WgradParams {
    const uint16_t* X;       // [K, ldx]        r (columns 0 .. rows_x): the contiguous index of `out`
    const uint16_t* Y;       // [K, ldy]        c (columns 0 .. rows_y): the row index of `out`
    float* out;              // [rows_y, ld]    out[c][r] (+)= sum_k X[k][r] Y[k][c]
    int64_t ldx, ldy, ld;
    int rows_x, rows_y, K;
    int first;               // store instead of add
};

struct WgradBatch {
    WgradParams p[kMaxBatch];
    BatchMap map;
};

template <class Core, bool GUARD>
__global__ __launch_bounds__(Core::kThreads) void wgrad_kernel(const WgradBatch b) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    extern __shared__ __align__(16) unsigned char smem[];
    int which, tr, tc, PR, PC;
    if (!b.map.locate(blockIdx.x, which, tr, tc, PR, PC)) return;
    const WgradParams& p = b.p[which];
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    int64_t step = 0;
    const uint16_t* warm = Core::kCanGuard ? nullptr
                                           : warm_line_kmajor(PR, PC, p.X, p.ldx, r0, tr, p.Y, p.ldy,
                                                              c0, tc, step, p.rows_x, p.rows_y);
    Core::template gemm<GUARD>(p.X, p.ldx, p.rows_x, p.Y, p.ldy, p.rows_y, p.K, r0, c0, smem, acc, warm,
                               step);
    accumulate_block_f32<Core, GUARD>(acc, p.out, p.ld, r0, c0, p.rows_x, p.rows_y, p.first != 0);
}

// out = sums (bf16 or fp32, overwrite or +=).  `sums` may alias `out` (fp32 overwrite mode).
template <bool OUT_F32, bool ACCUM>
__global__ void convert_sums_kernel(const float* sums, void* out, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
         i += (int64_t)gridDim.x * blockDim.x) {
        f32x4_t a = reinterpret_cast<const f32x4_t*>(sums)[i];
        if (OUT_F32) {
            f32x4_t* o = reinterpret_cast<f32x4_t*>(out) + i;
            if (ACCUM) a += *o;
            *o = a;
        } else {
            bf16x4_t* o = reinterpret_cast<bf16x4_t*>(out) + i;
            if (ACCUM) {
                const bf16x4_t old = *o;
#pragma unroll
                for (int x = 0; x < 4; ++x) a[x] += (float)old[x];
            }
            bf16x4_t r;
#pragma unroll
            for (int x = 0; x < 4; ++x) r[x] = (__bf16)a[x];
            *o = r;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static int prepare_mlp_kernels_on_current_device() {
    int rc = ALST_OK;
    auto acc = [&](int r) { if (r != ALST_OK) rc = r; };
    acc(allow_big_lds(linear_kernel<DirectCore, false>));
    acc(allow_big_lds(linear_chain_kernel, kChainLdsBytes));
    acc(allow_big_lds(linear_kernel<StagedCore, true>));
    acc(allow_big_lds(linear_kernel<MixedCore, false>));
    acc(allow_big_lds(linear_kernel<StagedMixedCore, true>));
    acc(allow_big_lds(gated_kernel<DirectCore, false, false>));
    acc(allow_big_lds(gated_kernel<StagedCore, true, false>));
    acc(allow_big_lds(gated_kernel<DirectCore, false, true>));
    acc(allow_big_lds(gated_kernel<DirectCore, false, false, true>));
    acc(allow_big_lds(gated_kernel<DirectCore, false, true, true>));
    acc(allow_big_lds(gated_chain_kernel<false, false>, kChainLdsBytes));
    acc(allow_big_lds(gated_chain_kernel<true, false>, kChainLdsBytes));
    acc(allow_big_lds(gated_chain_kernel<false, true>, kChainLdsBytes));
    acc(allow_big_lds(gated_chain_kernel<true, true>, kChainLdsBytes));
    acc(allow_big_lds(gated_kernel<StagedCore, true, true>));
    acc(allow_big_lds(wgrad_kernel<KMajorCore, false>));
    acc(allow_big_lds(wgrad_kernel<StagedKMajorCore, true>));
    return rc;
}
// Once per device, whatever the number of host threads that make their first call together.
static int prepare_mlp_kernels() {
    static std::once_flag once[kMaxDevices];
    static int results[kMaxDevices];
    const int dev = current_device_slot();
    if (dev < 0) return ALST_ERR_HIP;
    std::call_once(once[dev], [dev] { results[dev] = prepare_mlp_kernels_on_current_device(); });
    return results[dev];
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// One launch for the n products (n <= kMaxBatch).
static int launch_linear(const LinearParams* ps, int n, hipStream_t s) {
    LinearBatch b = {};
    b.map.n = n;
    bool direct = true;
    int64_t patches = 0;
    for (int i = 0; i < n; ++i) {
        const LinearParams& p = ps[i];
        b.p[i] = p;
        b.map.first_patch[i] = (int)patches;
        const int tiles_r = (p.rows_x + kBlockR - 1) / kBlockR, tiles_c = (p.rows_y + kBlockC - 1) / kBlockC;
        b.map.g[i] = choose_patches(tiles_r, tiles_c);
        patches += b.map.g[i].patches();
        // the unguarded core needs every extent block-aligned and writes every row it computes
        direct = direct && p.rows_x % kBlockR == 0 && p.rows_y % kBlockC == 0 && p.K % kBlockK == 0 &&
                 p.K >= kBlockK && p.rows_out >= p.rows_x && p.cols_out >= p.rows_y;
    }
    if (patches * 32 > 0x7fffff00) return ALST_ERR_SHAPE;
    for (int i = n; i <= kMaxBatch; ++i) b.map.first_patch[i] = (int)patches;
    const int blocks = grid_for_patches(patches);
    ProfScope pr(PROF_MLP_LINEAR, s);
    const bool mixed = ps[0].y_kmajor != 0;           // the products of one launch are of one kind
    // persistent workgroups that fetch their next block early: one K, whole pairs of k-steps
    bool chain = ps[0].K % (2 * kBlockK) == 0 && ps[0].K >= 4 * kBlockK;
    for (int i = 1; i < n; ++i) chain = chain && ps[i].K == ps[0].K;
    if (direct && mixed)
        hipLaunchKernelGGL((linear_kernel<MixedCore, false>), dim3((unsigned)blocks),
                           dim3(MixedCore::kThreads), kLdsBytes, s, b);
    else if (direct && chain)
        hipLaunchKernelGGL(linear_chain_kernel, dim3((unsigned)std::min(blocks, persistent_grid())),
                           dim3(DirectCore::kThreads), kChainLdsBytes, s, b, blocks);
    else if (direct)
        hipLaunchKernelGGL((linear_kernel<DirectCore, false>), dim3((unsigned)blocks),
                           dim3(DirectCore::kThreads), kLdsBytes, s, b);
    else if (mixed)
        hipLaunchKernelGGL((linear_kernel<StagedMixedCore, true>), dim3((unsigned)blocks),
                           dim3(StagedMixedCore::kThreads), kLdsBytes, s, b);
    else
        hipLaunchKernelGGL((linear_kernel<StagedCore, true>), dim3((unsigned)blocks),
                           dim3(StagedCore::kThreads), kLdsBytes, s, b);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

static int launch_linear(const LinearParams& p, hipStream_t s) { return launch_linear(&p, 1, s); }

static int launch_wgrad_batch(const WgradParams* ps, int n, bool direct, hipStream_t s) {
    WgradBatch b = {};
    b.map.n = n;
    int64_t patches = 0;
    for (int i = 0; i < n; ++i) {
        const WgradParams& p = ps[i];
        b.p[i] = p;
        b.map.first_patch[i] = (int)patches;
        const int tiles_r = (p.rows_x + kBlockR - 1) / kBlockR, tiles_c = (p.rows_y + kBlockC - 1) / kBlockC;
        b.map.g[i] = choose_patches(tiles_r, tiles_c);
        patches += b.map.g[i].patches();
    }
    if (patches * 32 > 0x7fffff00) return ALST_ERR_SHAPE;
    for (int i = n; i <= kMaxBatch; ++i) b.map.first_patch[i] = (int)patches;
    const int blocks = grid_for_patches(patches);
    ProfScope pr(PROF_MLP_WGRAD, s);
    if (direct)
        hipLaunchKernelGGL((wgrad_kernel<KMajorCore, false>), dim3((unsigned)blocks),
                           dim3(KMajorCore::kThreads), kLdsBytes, s, b);
    else
        hipLaunchKernelGGL((wgrad_kernel<StagedKMajorCore, true>), dim3((unsigned)blocks),
                           dim3(StagedKMajorCore::kThreads), kLdsBytes, s, b);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

// The n weight-gradient products (n <= kMaxBatch, all with the same K) in one launch.  The
// unguarded core needs K in whole k-steps (output extents that end inside a block are its
// business): the whole k-steps go to it and the K % 64 rows left over to a second, guarded launch.
static int launch_wgrad(const WgradParams* ps, int n, hipStream_t s) {
    const int K = ps[0].K, K_whole = K / kBlockK * kBlockK;
    if (K_whole == 0) return launch_wgrad_batch(ps, n, false, s);
    WgradParams part[kMaxBatch];
    for (int i = 0; i < n; ++i) { part[i] = ps[i]; part[i].K = K_whole; }
    int rc = launch_wgrad_batch(part, n, true, s);
    if (rc != ALST_OK || K_whole == K) return rc;
    for (int i = 0; i < n; ++i) {
        part[i].X += (int64_t)K_whole * ps[i].ldx;
        part[i].Y += (int64_t)K_whole * ps[i].ldy;
        part[i].K = K - K_whole;
        part[i].first = 0;
    }
    return launch_wgrad_batch(part, n, false, s);
}

static int launch_wgrad(const WgradParams& p, hipStream_t s) { return launch_wgrad(&p, 1, s); }

struct MlpProblem {
    const uint16_t *x, *Wg, *Wu, *Wd, *dy;
    uint16_t *y, *dx;
    void *dWg, *dWu, *dWd;
    int64_t N, H, I, tile;
    unsigned char* ws;
    uint32_t flags;
    hipStream_t stream;
};

static int validate_mlp(const MlpProblem& P, size_t workspace_bytes, bool backward) {
    if (!P.x || !P.Wg || !P.Wu || !P.Wd || !P.ws) return ALST_ERR_NULL;
    if (!backward && !P.y) return ALST_ERR_NULL;
    if (backward && (!P.dy || !P.dx || !P.dWg || !P.dWu || !P.dWd)) return ALST_ERR_NULL;
    if (P.flags & ~(ALST_FLAG_DW_FP32 | ALST_FLAG_DW_ACCUMULATE)) return ALST_ERR_UNSUPPORTED;
    if (P.N < 1 || P.H < 1 || P.I < 1 || P.tile < 1) return ALST_ERR_SHAPE;
    if (P.N > (int64_t)1 << 30 || P.H > (int64_t)1 << 20 || P.I > (int64_t)1 << 20) return ALST_ERR_SHAPE;
    if (P.H % 8 != 0 || P.I % 8 != 0) return ALST_ERR_ALIGN;
    const void* ptrs[] = {P.x, P.Wg, P.Wu, P.Wd, P.ws, P.y, P.dy, P.dx, P.dWg, P.dWu, P.dWd};
    for (const void* q : ptrs)
        if (q && !aligned16(q)) return ALST_ERR_ALIGN;
    const MlpLayout L = make_mlp_layout(P.N, P.H, P.I, P.tile, backward, P.flags);
    // every launch must fit its grid (the widest are [T, 2I] and [2I, H] outputs)
    if (!checked_grid(L.Tp / kBlockR, (2 * P.I + kBlockC - 1) / kBlockC) ||
        !checked_grid((P.I + kBlockR - 1) / kBlockR, (P.H + kBlockC - 1) / kBlockC))
        return ALST_ERR_SHAPE;
    if (workspace_bytes < L.total) return ALST_ERR_WORKSPACE;
    return ALST_OK;
}

// a = silu(x_t Wg^T) * (x_t Wu^T) for the tile's T_cur rows (rows up to Tr come out as zeros);
// backward (da given): also [dg | du].
static int launch_gated(const MlpProblem& P, const uint16_t* x_t, int T_cur, int Tr,
                        const uint16_t* da, uint16_t* a, uint16_t* dgu, hipStream_t s) {
    GatedParams gp = {};
    gp.X = x_t; gp.ldx = P.H; gp.rows_x = T_cur; gp.K = (int)P.H;
    gp.Wg = P.Wg; gp.Wu = P.Wu; gp.ldw = P.H; gp.I = (int)P.I;
    gp.da = da; gp.a = a; gp.dgu = dgu; gp.rows_out = Tr;
    gp.grid = choose_patches(Tr / kBlockR, (int)((P.I + 127) / 128));
    const int blocks = grid_for_patches(gp.grid.patches());
    // the unguarded core needs whole blocks of rows and whole k-steps; an I that ends inside a
    // block's 128 columns is handled by its epilogue
    const bool direct = T_cur % kBlockR == 0 && P.H % kBlockK == 0;
    const bool cguard = P.I % 128 != 0;
    // persistent workgroups that fetch their next block early: whole pairs of k-steps
    const bool chain = direct && P.H % (2 * kBlockK) == 0 && P.H >= 4 * kBlockK;
    ProfScope pr(PROF_MLP_LINEAR, s);
    if (chain) {
        const dim3 grid((unsigned)std::min(blocks, persistent_grid())), block(DirectCore::kThreads);
        if (cguard && da) hipLaunchKernelGGL((gated_chain_kernel<true, true>), grid, block, kChainLdsBytes, s, gp, blocks);
        else if (cguard) hipLaunchKernelGGL((gated_chain_kernel<false, true>), grid, block, kChainLdsBytes, s, gp, blocks);
        else if (da) hipLaunchKernelGGL((gated_chain_kernel<true, false>), grid, block, kChainLdsBytes, s, gp, blocks);
        else hipLaunchKernelGGL((gated_chain_kernel<false, false>), grid, block, kChainLdsBytes, s, gp, blocks);
    } else if (direct && cguard && da)
        hipLaunchKernelGGL((gated_kernel<DirectCore, false, true, true>), dim3((unsigned)blocks),
                           dim3(DirectCore::kThreads), kLdsBytes, s, gp);
    else if (direct && cguard)
        hipLaunchKernelGGL((gated_kernel<DirectCore, false, false, true>), dim3((unsigned)blocks),
                           dim3(DirectCore::kThreads), kLdsBytes, s, gp);
    else if (direct && da)
        hipLaunchKernelGGL((gated_kernel<DirectCore, false, true>), dim3((unsigned)blocks),
                           dim3(DirectCore::kThreads), kLdsBytes, s, gp);
    else if (direct)
        hipLaunchKernelGGL((gated_kernel<DirectCore, false, false>), dim3((unsigned)blocks),
                           dim3(DirectCore::kThreads), kLdsBytes, s, gp);
    else if (da)
        hipLaunchKernelGGL((gated_kernel<StagedCore, true, true>), dim3((unsigned)blocks),
                           dim3(StagedCore::kThreads), kLdsBytes, s, gp);
    else
        hipLaunchKernelGGL((gated_kernel<StagedCore, true, false>), dim3((unsigned)blocks),
                           dim3(StagedCore::kThreads), kLdsBytes, s, gp);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

static int run_mlp_forward(const MlpProblem& P) {
    int rc = prepare_mlp_kernels();
    if (rc != ALST_OK) return rc;
    const MlpLayout L = make_mlp_layout(P.N, P.H, P.I, P.tile, false, P.flags);
    hipStream_t s = P.stream;
    uint16_t* a = reinterpret_cast<uint16_t*>(P.ws + L.a);
    const int H = (int)P.H, I = (int)P.I;
    const int64_t T = P.tile < P.N ? P.tile : P.N;
    const int64_t ntiles = (P.N + T - 1) / T;
    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t i0 = t * T;
        const int T_cur = (int)((P.N - i0) < T ? (P.N - i0) : T);
        const int Tr = (T_cur + kBlockR - 1) / kBlockR * kBlockR;
        rc = launch_gated(P, P.x + i0 * P.H, T_cur, Tr, nullptr, a, nullptr, s);
        if (rc != ALST_OK) return rc;
        LinearParams lp = {};
        lp.X = a; lp.ldx = I; lp.rows_x = Tr; lp.K = I;
        lp.Y = P.Wd; lp.ldy = I; lp.rows_y = H;
        lp.D = P.y + i0 * P.H; lp.ldd = H; lp.rows_out = T_cur; lp.cols_out = H;
        rc = launch_linear(lp, s);
        if (rc != ALST_OK) return rc;
    }
    return ALST_OK;
}

template <bool F32, bool ACC>
static void launch_convert(const float* sums, void* out, int64_t n, hipStream_t s) {
    const int64_t n4 = n / 4;
    int blocks = (int)((n4 + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL((convert_sums_kernel<F32, ACC>), dim3(blocks), dim3(256), 0, s, sums, out, n4);
}

static int run_mlp_backward(const MlpProblem& P) {
    int rc = prepare_mlp_kernels();
    if (rc != ALST_OK) return rc;
    const MlpLayout L = make_mlp_layout(P.N, P.H, P.I, P.tile, true, P.flags);
    hipStream_t s = P.stream;
    uint16_t* a = reinterpret_cast<uint16_t*>(P.ws + L.a);
    uint16_t* da = reinterpret_cast<uint16_t*>(P.ws + L.da);
    uint16_t* dgu = reinterpret_cast<uint16_t*>(P.ws + L.dgu);
    const bool f32 = P.flags & ALST_FLAG_DW_FP32, accum = P.flags & ALST_FLAG_DW_ACCUMULATE;
    const bool in_out = f32 && !accum;
    float* acc_g = in_out ? reinterpret_cast<float*>(P.dWg) : reinterpret_cast<float*>(P.ws + L.acc_g);
    float* acc_u = in_out ? reinterpret_cast<float*>(P.dWu) : reinterpret_cast<float*>(P.ws + L.acc_u);
    float* acc_d = in_out ? reinterpret_cast<float*>(P.dWd) : reinterpret_cast<float*>(P.ws + L.acc_d);
    const int H = (int)P.H, I = (int)P.I;
    const int64_t I2 = 2 * (int64_t)I;

    uint16_t* wdt = reinterpret_cast<uint16_t*>(P.ws + L.wdt);
    uint16_t* wgut = reinterpret_cast<uint16_t*>(P.ws + L.wgut);
    if (L.weights_t) {
        ProfScope ps(PROF_MLP_OTHER, s);
        const dim3 gd((unsigned)((H + 63) / 64), (unsigned)((I + 63) / 64)), gi(gd.y, gd.x);
        hipLaunchKernelGGL(transpose_bf16_kernel, gd, dim3(256), 0, s, P.Wd, H, I, (int64_t)I, wdt, (int64_t)H);
        hipLaunchKernelGGL(transpose_bf16_kernel, gi, dim3(256), 0, s, P.Wg, I, H, (int64_t)H, wgut, I2);
        hipLaunchKernelGGL(transpose_bf16_kernel, gi, dim3(256), 0, s, P.Wu, I, H, (int64_t)H, wgut + I, I2);
        ALST_HIP(hipGetLastError());
    }

    const int64_t T = P.tile < P.N ? P.tile : P.N;
    const int64_t ntiles = (P.N + T - 1) / T;
    int kofs = 0;                                   // rows of the group so far
    int64_t group_row0 = 0;                         // first row of the group in x and dy
    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t i0 = t * T;
        const int T_cur = (int)((P.N - i0) < T ? (P.N - i0) : T);
        const int Tr = (T_cur + kBlockR - 1) / kBlockR * kBlockR;
        const int slot = (int)(t % L.g);
        if (slot == 0) { kofs = 0; group_row0 = i0; }
        const uint16_t* x_t = P.x + i0 * P.H;
        const uint16_t* dy_t = P.dy + i0 * P.H;
        // the tile's rows of a and [dg | du] sit behind those of the group's earlier tiles (rows
        // T_cur .. Tr come out as zeros and are overwritten by the next tile)
        uint16_t* a_t = a + (int64_t)kofs * I;
        uint16_t* dgu_t = dgu + (int64_t)kofs * I2;

        {   // da = dy_t Wd (contraction over H), then g and u again with a, dg, du made in the epilogue
            LinearParams lp = {};
            lp.X = dy_t; lp.ldx = H; lp.rows_x = T_cur; lp.K = H;
            if (L.weights_t) { lp.Y = wdt; lp.ldy = H; lp.rows_y = I; }            // Wd^T [I, H]
            else { lp.Y = P.Wd; lp.ldy = I; lp.rows_y = I; lp.y_kmajor = 1; }      // Wd [H, I]: k = h
            lp.D = da; lp.ldd = I; lp.rows_out = Tr; lp.cols_out = I;
            rc = launch_linear(lp, s);
            if (rc == ALST_OK) rc = launch_gated(P, x_t, T_cur, Tr, da, a_t, dgu_t, s);
            if (rc != ALST_OK) return rc;
        }
        {   // dx = dg Wg + du Wu
            LinearParams lp = {};
            lp.X = dgu_t; lp.ldx = I2; lp.rows_x = Tr;
            if (L.weights_t) {
                // one contraction over the 2 I columns of [dg | du] against [Wg | Wu]^T [H, 2 I]
                lp.K = (int)I2; lp.Y = wgut; lp.ldy = I2; lp.rows_y = H;
            } else {
                // two contractions over I summed in the accumulators, the weights as they are
                lp.K = I; lp.Y = P.Wg; lp.ldy = H; lp.rows_y = H; lp.y_kmajor = 1;     // Wg [I, H]: k = i
                lp.X2 = dgu_t + I; lp.Y2 = P.Wu;
            }
            lp.D = P.dx + i0 * P.H; lp.ldd = H; lp.rows_out = T_cur; lp.cols_out = H;
            rc = launch_linear(lp, s);
            if (rc != ALST_OK) return rc;
        }
        kofs += T_cur;
        if (slot == L.g - 1 || t == ntiles - 1) {       // the group is complete
            const int first = t < L.g;
            const uint16_t* x_g = P.x + group_row0 * P.H;
            const uint16_t* dy_g = P.dy + group_row0 * P.H;
            WgradParams wp[kMaxBatch] = {};
            wp[0].K = kofs; wp[0].first = first;
            wp[0].X = x_g; wp[0].ldx = H; wp[0].rows_x = H; wp[0].ld = H;
            wp[0].Y = dgu; wp[0].ldy = I2; wp[0].rows_y = I; wp[0].out = acc_g;      // dWg[i][h]
            wp[1] = wp[0];
            wp[1].Y = dgu + I; wp[1].out = acc_u;                                    // dWu[i][h]
            wp[2] = wp[0];
            wp[2].X = a; wp[2].ldx = I; wp[2].rows_x = I; wp[2].ld = I;
            wp[2].Y = dy_g; wp[2].ldy = H; wp[2].rows_y = H; wp[2].out = acc_d;      // dWd[h][i]
            rc = launch_wgrad(wp, 3, s);                                             // one launch
            if (rc != ALST_OK) return rc;
        }
    }
    if (!in_out) {
        ProfScope ps(PROF_MLP_OTHER, s);
        const int64_t n = P.I * P.H;
        float* sums[3] = {acc_g, acc_u, acc_d};
        void* outs[3] = {P.dWg, P.dWu, P.dWd};
        for (int k = 0; k < 3; ++k) {
            if (f32) launch_convert<true, true>(sums[k], outs[k], n, s);          // fp32 +=
            else if (accum) launch_convert<false, true>(sums[k], outs[k], n, s);
            else launch_convert<false, false>(sums[k], outs[k], n, s);
        }
        ALST_HIP(hipGetLastError());
    }
    return ALST_OK;
}

// ---------------------------------------------------------------------------------------------
// the single tiled linear layer: y = x W^T, dx = dy W, dW = dy^T x
// ---------------------------------------------------------------------------------------------
struct LinLayout {
    int64_t Tp;
    int g;                 // tiles per weight-gradient group
    size_t acc, wt, total;
    bool weight_t;         // backward multiplies dy by a transposed copy of W
};

static LinLayout make_lin_layout(int64_t N, int64_t K, int64_t M, int64_t tile, bool backward,
                                 uint32_t flags) {
    LinLayout L = {};
    const int64_t T = tile < N ? tile : N;
    L.Tp = (T + 255) / 256 * 256;
    int64_t g = kMlpGroupRows / L.Tp;
    L.g = (int)(g < 1 ? 1 : (g > kMlpGroupMax ? kMlpGroupMax : g));
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    if (backward) {
        const bool in_out = (flags & ALST_FLAG_DW_FP32) && !(flags & ALST_FLAG_DW_ACCUMULATE);
        L.acc = take(in_out ? 0 : (size_t)M * K * 4);
        // W transposed [K, M], made once per call: dx = dy W then reads both operands along their
        // rows (the fastest layout of the block GEMM).  For M a multiple of 64; else W is read
        // as it is.
        L.weight_t = M % kBlockK == 0;
        L.wt = take(L.weight_t ? (size_t)K * M * 2 : 0);
    }
    L.total = o;
    return L;
}

struct LinProblem {
    const uint16_t *x, *W, *dy;
    uint16_t *y, *dx;
    void* dW;
    int64_t N, K, M, tile;
    unsigned char* ws;
    uint32_t flags;
    hipStream_t stream;
};

static int validate_lin(const LinProblem& P, size_t workspace_bytes, bool backward) {
    if (!P.x || !P.W) return ALST_ERR_NULL;
    if (!backward && !P.y) return ALST_ERR_NULL;
    if (backward && (!P.dy || !P.dx || !P.dW)) return ALST_ERR_NULL;
    if (P.flags & ~(ALST_FLAG_DW_FP32 | ALST_FLAG_DW_ACCUMULATE)) return ALST_ERR_UNSUPPORTED;
    if (P.N < 1 || P.K < 1 || P.M < 1 || P.tile < 1) return ALST_ERR_SHAPE;
    if (P.N > (int64_t)1 << 30 || P.K > (int64_t)1 << 20 || P.M > (int64_t)1 << 24) return ALST_ERR_SHAPE;
    // (forward needs no scratch)
    if (make_lin_layout(P.N, P.K, P.M, P.tile, backward, P.flags).total > 0 && !P.ws) return ALST_ERR_NULL;
    if (P.K % 8 != 0 || P.M % 8 != 0) return ALST_ERR_ALIGN;
    const void* ptrs[] = {P.x, P.W, P.dy, P.y, P.dx, P.dW, P.ws};
    for (const void* q : ptrs)
        if (q && !aligned16(q)) return ALST_ERR_ALIGN;
    const LinLayout L = make_lin_layout(P.N, P.K, P.M, P.tile, backward, P.flags);
    if (!checked_grid(L.Tp / kBlockR, (P.M + kBlockC - 1) / kBlockC) ||
        !checked_grid((P.K + kBlockR - 1) / kBlockR, (P.M + kBlockC - 1) / kBlockC))
        return ALST_ERR_SHAPE;
    if (workspace_bytes < L.total) return ALST_ERR_WORKSPACE;
    return ALST_OK;
}

static int run_lin_forward(const LinProblem& P) {
    int rc = prepare_mlp_kernels();
    if (rc != ALST_OK) return rc;
    const int64_t T = P.tile < P.N ? P.tile : P.N;
    const int64_t ntiles = (P.N + T - 1) / T;
    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t i0 = t * T;
        const int T_cur = (int)((P.N - i0) < T ? (P.N - i0) : T);
        LinearParams lp = {};
        lp.X = P.x + i0 * P.K; lp.ldx = P.K; lp.rows_x = T_cur; lp.K = (int)P.K;
        lp.Y = P.W; lp.ldy = P.K; lp.rows_y = (int)P.M;
        lp.D = P.y + i0 * P.M; lp.ldd = P.M; lp.rows_out = T_cur; lp.cols_out = (int)P.M;
        rc = launch_linear(lp, P.stream);
        if (rc != ALST_OK) return rc;
    }
    return ALST_OK;
}

static int run_lin_backward(const LinProblem& P) {
    int rc = prepare_mlp_kernels();
    if (rc != ALST_OK) return rc;
    const LinLayout L = make_lin_layout(P.N, P.K, P.M, P.tile, true, P.flags);
    hipStream_t s = P.stream;
    const bool f32 = P.flags & ALST_FLAG_DW_FP32, accum = P.flags & ALST_FLAG_DW_ACCUMULATE;
    const bool in_out = f32 && !accum;
    float* acc = in_out ? reinterpret_cast<float*>(P.dW) : reinterpret_cast<float*>(P.ws + L.acc);
    const int K = (int)P.K, M = (int)P.M;
    const int64_t T = P.tile < P.N ? P.tile : P.N;
    const int64_t ntiles = (P.N + T - 1) / T;
    uint16_t* wt = reinterpret_cast<uint16_t*>(P.ws + L.wt);
    if (L.weight_t) {
        ProfScope ps(PROF_MLP_OTHER, s);
        hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((M + 63) / 64), (unsigned)((K + 63) / 64)),
                           dim3(256), 0, s, P.W, M, K, (int64_t)K, wt, (int64_t)M);
        ALST_HIP(hipGetLastError());
    }
    int kofs = 0;                                   // rows of the group so far
    int64_t group_row0 = 0;
    for (int64_t t = 0; t < ntiles; ++t) {
        const int64_t i0 = t * T;
        const int T_cur = (int)((P.N - i0) < T ? (P.N - i0) : T);
        const int slot = (int)(t % L.g);
        if (slot == 0) { kofs = 0; group_row0 = i0; }
        LinearParams lp = {};
        lp.X = P.dy + i0 * P.M; lp.ldx = M; lp.rows_x = T_cur; lp.K = M;
        if (L.weight_t) { lp.Y = wt; lp.ldy = M; lp.rows_y = K; }         // W^T [K, M]
        else { lp.Y = P.W; lp.ldy = K; lp.rows_y = K; lp.y_kmajor = 1; }  // W [M, K]: k = m
        lp.D = P.dx + i0 * P.K; lp.ldd = K; lp.rows_out = T_cur; lp.cols_out = K;
        rc = launch_linear(lp, s);
        if (rc != ALST_OK) return rc;
        kofs += T_cur;
        if (slot == L.g - 1 || t == ntiles - 1) {
            // dW[m][k] += sum over the group's rows of dy[t][m] x[t][k]: both operands are read
            // from the caller's arrays as they are
            WgradParams wp = {};
            wp.X = P.x + group_row0 * P.K; wp.ldx = K; wp.rows_x = K;
            wp.Y = P.dy + group_row0 * P.M; wp.ldy = M; wp.rows_y = M;
            wp.K = kofs; wp.out = acc; wp.ld = K; wp.first = t < L.g;
            rc = launch_wgrad(wp, s);
            if (rc != ALST_OK) return rc;
        }
    }
    if (!in_out) {
        ProfScope ps(PROF_MLP_OTHER, s);
        const int64_t n = P.M * P.K;
        if (f32) launch_convert<true, true>(acc, P.dW, n, s);
        else if (accum) launch_convert<false, true>(acc, P.dW, n, s);
        else launch_convert<false, false>(acc, P.dW, n, s);
        ALST_HIP(hipGetLastError());
    }
    return ALST_OK;
}

}  // namespace alst

using namespace alst;

extern "C" {

size_t alst_tiled_mlp_workspace_bytes(int64_t N, int64_t H, int64_t I, int64_t tile, int backward,
                                      uint32_t flags) {
    if (N < 1 || H < 1 || I < 1 || tile < 1) return 0;
    if (N > (int64_t)1 << 30 || H > (int64_t)1 << 20 || I > (int64_t)1 << 20) return 0;
    return make_mlp_layout(N, H, I, tile, backward != 0, flags).total;
}

int alst_tiled_mlp_forward(const void* x, const void* Wg, const void* Wu, const void* Wd, int64_t N,
                           int64_t H, int64_t I, int64_t tile, void* y, void* workspace,
                           size_t workspace_bytes, uint32_t flags, void* stream) {
    MlpProblem P = {};
    P.x = (const uint16_t*)x; P.Wg = (const uint16_t*)Wg; P.Wu = (const uint16_t*)Wu;
    P.Wd = (const uint16_t*)Wd; P.y = (uint16_t*)y;
    P.N = N; P.H = H; P.I = I; P.tile = tile;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate_mlp(P, workspace_bytes, false);
    if (rc != ALST_OK) return rc;
    return run_mlp_forward(P);
}

int alst_tiled_mlp_backward(const void* x, const void* Wg, const void* Wu, const void* Wd,
                            const void* dy, int64_t N, int64_t H, int64_t I, int64_t tile, void* dx,
                            void* dWg, void* dWu, void* dWd, void* workspace, size_t workspace_bytes,
                            uint32_t flags, void* stream) {
    MlpProblem P = {};
    P.x = (const uint16_t*)x; P.Wg = (const uint16_t*)Wg; P.Wu = (const uint16_t*)Wu;
    P.Wd = (const uint16_t*)Wd; P.dy = (const uint16_t*)dy; P.dx = (uint16_t*)dx;
    P.dWg = dWg; P.dWu = dWu; P.dWd = dWd;
    P.N = N; P.H = H; P.I = I; P.tile = tile;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate_mlp(P, workspace_bytes, true);
    if (rc != ALST_OK) return rc;
    return run_mlp_backward(P);
}

size_t alst_tiled_linear_workspace_bytes(int64_t N, int64_t K, int64_t M, int64_t tile, int backward,
                                         uint32_t flags) {
    if (N < 1 || K < 1 || M < 1 || tile < 1) return 0;
    if (N > (int64_t)1 << 30 || K > (int64_t)1 << 20 || M > (int64_t)1 << 24) return 0;
    return make_lin_layout(N, K, M, tile, backward != 0, flags).total;
}

int alst_tiled_linear_forward(const void* x, const void* W, int64_t N, int64_t K, int64_t M,
                              int64_t tile, void* y, void* workspace, size_t workspace_bytes,
                              uint32_t flags, void* stream) {
    LinProblem P = {};
    P.x = (const uint16_t*)x; P.W = (const uint16_t*)W; P.y = (uint16_t*)y;
    P.N = N; P.K = K; P.M = M; P.tile = tile;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate_lin(P, workspace_bytes, false);
    if (rc != ALST_OK) return rc;
    return run_lin_forward(P);
}

int alst_tiled_linear_backward(const void* x, const void* W, const void* dy, int64_t N, int64_t K,
                               int64_t M, int64_t tile, void* dx, void* dW, void* workspace,
                               size_t workspace_bytes, uint32_t flags, void* stream) {
    LinProblem P = {};
    P.x = (const uint16_t*)x; P.W = (const uint16_t*)W; P.dy = (const uint16_t*)dy;
    P.dx = (uint16_t*)dx; P.dW = dW;
    P.N = N; P.K = K; P.M = M; P.tile = tile;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate_lin(P, workspace_bytes, true);
    if (rc != ALST_OK) return rc;
    return run_lin_backward(P);
}

}  // extern "C"

