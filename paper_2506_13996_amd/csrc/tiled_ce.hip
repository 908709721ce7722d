// Sequence-tiled LM-head projection + cross-entropy for gfx950: kernels and the C ABI (alst.h).
//
// Per sequence tile of T rows (paper, section "Sequence Tiling for Reducing Activation Memory
// Footprint": forward and backward of each logits shard are done together and the shard's
// intermediates are dropped before the next shard):
//
//   0. tile_info /       rows whose label is ignored take no part in the loss or in either gradient:
//      gather_rows       once per call the valid rows are numbered densely in sequence order
//                        (block_count / block_offsets / scatter_index, which also zero-fill the
//                        dHidden rows and loss terms of ignored tokens), and a tile is T
//                        consecutive dense rows, gathered into a dense [T, H] copy (behind the
//                        rows of the earlier tiles of its dW group).  Their number
//                        M lives on the device: the host walks ceil(N / T) tiles and the kernels
//                        of a tile beyond the dense rows leave at once, so nothing waits for the
//                        host.
//   1. logits_kernel     Z = H_c W^T in 256x256 blocks, fp32 accumulators.  The logits never
//                        leave the registers: the epilogue picks out the label logit, writes
//                        e = exp(z - ref_i) as bf16 to a [T, V] scratch ("stash", also laid out
//                        per dW group) and reduces each row over the block's columns to
//                        (max, sum e) partials per 128-column group.  ref_i is ONE reference per
//                        row (0 to begin with), so a row's softmax is e / S_i with S_i = sum_v e:
//                        the scale is a per-row scalar that the consumers of the stash apply.
//   2. row_finish        partials -> S_i, lse_i = ref_i + log S_i, per-row loss; the label entry of
//                        the stash becomes e - S_i (so that e' / S_i = p - onehot), and the row's
//                        dense hidden row is scaled by 1 / S_i in place (the dW operand).  A row
//                        whose S_i left the safe range of the bf16 / fp32 exponents (logits
//                        beyond about +-40) is redone with ref_i = its exact maximum: a second,
//                        conditional launch of 1. and 2. whose workgroups leave at once when no
//                        row of the tile asked for it.
//   3. dhidden_kernel    dH_i = (g/M) (1/S_i) e'_i W   (contraction over V), rows scattered back
//   4. dw_kernel         acc += (H_c / S)^T e'         once per group of tiles (contraction over
//                        the group's dense rows, fp32)
//
// After the last tile: loss = sum(per-row loss) / M in a fixed order, dW = (g/M) acc.
// The contractions share the block GEMM of gemm_tile.h: logits and dHidden with both operands
// k-contiguous (dHidden against a copy of W transposed once per call), dW with both operands
// k-major (the group's dense hidden rows and dZ rows as they are).  No per-tile array is
// transposed.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <mutex>

#include "../../include/alst.h"
#include "gemm_tile.h"
#include "common.h"

namespace alst {

// ---------------------------------------------------------------------------------------------
// workspace
// ---------------------------------------------------------------------------------------------
struct Header {
    int status;            // alst_status set by kernels
    int pad0;
    long long n_valid;     // M
    float inv;             // g / M (0 when M == 0)
    float pad1;
    double loss_sum;
};

// What tile_info_kernel leaves for the other kernels of a tile.
struct TileInfo {
    int Tc;                // rows of the tile that take part (valid label)
    int Trc;               // Tc rounded up to the block height (256)
    int Tkc;               // Tc rounded up to the k-step (64)
    int kofs;              // where the tile's dense rows start along k in the dW group buffers
    int splits;            // dHidden: ranges the contraction over V is cut into for this tile
    int ksteps;            //          k-steps of 64 per range (the last range may be shorter)
    int redo;              // set by row_finish: some row of the tile needs the second logits pass
    int pad;
};

// dW is accumulated into the fp32 [V, H] sums once per GROUP of consecutive tiles: the dense
// hidden rows and dZ rows of the group's tiles are kept one behind the other and one dW GEMM
// contracts over all of them, so the read-modify-write of the 4*V*H-byte accumulator and the
// GEMM's epilogue are paid once per group instead of once per tile.  The group spans about
// kDwGroupRows rows.
constexpr int kDwGroupRows = 16384;
constexpr int kDwGroupMax = 8;
// ALST_FLAG_TILE_SCRATCH (and the forward-only layout, which keeps no dZ at all): groups of one tile.
static inline int dw_group_size(int64_t Tp, uint32_t flags) {
    if (flags & (ALST_FLAG_TILE_SCRATCH | ALST_FLAG_FORWARD_ONLY)) return 1;
    int64_t g = kDwGroupRows / Tp;
    return (int)(g < 1 ? 1 : (g > kDwGroupMax ? kDwGroupMax : g));
}
constexpr uint32_t kKnownFlags = ALST_FLAG_DW_FP32 | ALST_FLAG_DW_ACCUMULATE | ALST_FLAG_REDUCE_SUM |
                                 ALST_FLAG_TILE_SCRATCH | ALST_FLAG_FORWARD_ONLY;

constexpr int kScanThreads = 1024;   // rows per block of the compaction kernels

struct Layout {
    int64_t Tp, Vp, ng;    // padded tile rows, padded vocabulary, 128-column groups
    int64_t Hk;            // row pitch of the dense hidden copy: H rounded up to whole k-steps
    int g;                 // tiles per dW group
    int64_t Kg;            // dense rows a group can hold: g * Tp
    int dh_PR, dh_PC;      // dHidden: patch shape of the block -> tile mapping
    int64_t dh_patches;    //          most patches (over all ranges) a tile of any number of rows needs
    int64_t dh_part_rows;  //          most rows of fp32 partial products (0: never cut)
    size_t header, tinfo, loss_rows, lse, idx, block_cnt, block_ofs, zlabel, yc, ref, frow, rowstate,
        pm, ps, hc, stash, wt, part, acc, total;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// dHidden has (rows / 256) * (H / 256) output blocks for a tile of `rows` dense rows (a multiple
// of 256).  Picks the number of ranges (1..8) the contraction over V is cut into so that the
// workgroups fill the 256 compute units of the chip most evenly (ties: fewest ranges), each range
// keeping at least 64 k-steps.  The tile's row count is known on the device only, so
// tile_info_kernel makes the choice; the host evaluates the same function for every possible row
// count to size the launch and the buffer of partial products.
constexpr int kComputeUnits = 256;
// part_rows_cap: the ranges' fp32 partial products (splits * rows rows) must fit that many rows
// (0: no limit).
__host__ __device__ inline void dhidden_splits(int64_t rows, int64_t H, int64_t V, int64_t part_rows_cap,
                                               int& splits, int& ksteps) {
    const int64_t blocks = (rows / kBlockR) * ((H + kBlockC - 1) / kBlockC);
    const int KT = (int)((V + kBlockK - 1) / kBlockK);
    int64_t best_wg = 0, best_slots = 1;               // fill = best_wg / best_slots
    splits = 1;
    // with 16 or more rounds of workgroups the chip is filled to 16/17 or better as it is (and the
    // products below stay small)
    const int sp_max = blocks >= 16 * kComputeUnits ? 1 : 8;
    for (int sp = 1; sp <= sp_max; ++sp) {
        const int per = (KT + sp - 1) / sp;
        if (sp > 1 && (per < 64 || (int64_t)(sp - 1) * per >= KT)) break;
        if (sp > 1 && part_rows_cap > 0 && sp * rows > part_rows_cap) break;
        const int64_t wg = blocks * sp;
        const int64_t slots = (wg + kComputeUnits - 1) / kComputeUnits * kComputeUnits;
        if (wg * best_slots > best_wg * slots) { best_wg = wg; best_slots = slots; splits = sp; }
    }
    ksteps = (KT + splits - 1) / splits;
}

static Layout make_layout(int64_t N, int64_t H, int64_t V, int64_t tile, uint32_t flags) {
    Layout L;
    const int64_t T = tile < N ? tile : N;
    L.Tp = (T + 255) / 256 * 256;
    L.Vp = (V + 255) / 256 * 256;
    L.ng = L.Vp / 128;
    L.Hk = (H + kBlockK - 1) / kBlockK * kBlockK;
    L.g = dw_group_size(L.Tp, flags);
    L.Kg = (int64_t)L.g * L.Tp;
    const bool fwd_only = flags & ALST_FLAG_FORWARD_ONLY;     // no dZ rows, partial products, dW sums
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.header = take(sizeof(Header));
    L.tinfo = take(sizeof(TileInfo) * kDwGroupMax);
    // the O(N) part: 12 bytes per row + 12 bytes per kScanThreads rows
    const size_t nblocks = ((size_t)N + kScanThreads - 1) / kScanThreads;
    L.loss_rows = take((size_t)N * 4);
    L.lse = take((size_t)N * 4);
    L.idx = take((size_t)N * 4);
    L.block_cnt = take(nblocks * 4);
    L.block_ofs = take(nblocks * 8);
    L.zlabel = take((size_t)L.Tp * 4);
    L.yc = take((size_t)L.Tp * 4);
    L.ref = take((size_t)L.Tp * 4);
    L.frow = take((size_t)L.Tp * 4);
    L.rowstate = take((size_t)L.Tp * 4);
    L.pm = take((size_t)L.ng * L.Tp * 4);
    L.ps = take((size_t)L.ng * L.Tp * 4);
    // hc and stash hold the dense rows of the whole group, each tile at its k offset: they are
    // the two operands of the group's dW product as they are (k = dense row, the slow index)
    L.hc = take((size_t)L.Kg * L.Hk * 2);
    L.stash = take(fwd_only ? 0 : (size_t)L.Kg * L.Vp * 2);
    // W transposed, [H, Vp] with zeros beyond V: the second operand of dH = dZ W, k-contiguous
    L.wt = take(fwd_only ? 0 : (size_t)H * L.Vp * 2);
    {   // dHidden: the launch and the partial products are sized for the worst tile
        const PatchGrid pg = choose_patches((int)(L.Tp / kBlockR), (int)((H + kBlockC - 1) / kBlockC));
        L.dh_PR = pg.PR; L.dh_PC = pg.PC;
        // partial products: what a full tile needs, and no less than one tile's rows, so that a
        // smaller last tile may be cut into more ranges than a full one
        int sp_full, ks;
        dhidden_splits(L.Tp, H, V, 0, sp_full, ks);
        L.dh_part_rows = (int64_t)sp_full * L.Tp;
        L.dh_patches = 0;
        // (beyond 4096 row blocks per tile only the full tile is looked at; tile_info_kernel then
        // keeps a smaller tile's choice within these bounds)
        const int64_t rb_max = L.Tp / kBlockR, rb_lo = rb_max > 4096 ? rb_max : 1;
        for (int64_t rb = rb_lo; rb <= rb_max; ++rb) {
            int sp;
            dhidden_splits(rb * kBlockR, H, V, L.dh_part_rows, sp, ks);
            const PatchGrid g = {(int)rb, pg.tiles_c, pg.PR, pg.PC};
            const int64_t patches = g.patches64() * sp;
            if (patches > L.dh_patches) L.dh_patches = patches;
        }
    }
    L.part = take(fwd_only ? 0 : (size_t)L.dh_part_rows * H * 4);
    const bool acc_in_dw = (flags & ALST_FLAG_DW_FP32) && !(flags & ALST_FLAG_DW_ACCUMULATE);
    L.acc = take(acc_in_dw || fwd_only ? 0 : (size_t)V * H * 4);
    L.total = o;
    return L;
}

// ---------------------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------------------
__global__ void init_header_kernel(Header* h) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        h->status = 0;
        h->n_valid = 0;
        h->inv = 0.f;
        h->loss_sum = 0.0;
    }
}

__device__ __forceinline__ bool label_valid(int y, int ignore_index, int V) {
    return y != ignore_index && y >= 0 && y < V;
}

// Row compaction of the whole sequence: idx[j] = row of the j-th token with a valid label, in
// sequence order.  Three small kernels over blocks of kScanThreads rows:
//   block_count_kernel   valid rows per block
//   block_offsets_kernel exclusive scan of the block counts (one workgroup), M = their sum
//   scatter_index_kernel rank inside the block + block offset -> idx; rows that take no part get
//                        loss term 0 and lse 0 (forward) and a zero dHidden row (backward).
// The dense rows are then cut into tiles of T rows: tile t = dense rows [t T, min((t + 1) T, M)).
__device__ __forceinline__ int block_rank(bool valid, int* wave_total, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long mask = __ballot(valid);
    const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        const int c = wave_total[w];
        if (w < wave) before += c;
        total += c;
    }
    __syncthreads();
    return before + below;
}

__global__ __launch_bounds__(kScanThreads) void block_count_kernel(
    const int32_t* __restrict__ labels, int64_t N, int ignore_index, int V,
    int32_t* __restrict__ block_cnt, Header* h) {
    __shared__ int wave_total[kScanThreads / 64];
    const int64_t i = (int64_t)blockIdx.x * kScanThreads + threadIdx.x;
    const int y = i < N ? labels[i] : ignore_index;
    const bool valid = i < N && label_valid(y, ignore_index, V);
    if (i < N && y != ignore_index && !valid) atomicMax(&h->status, (int)ALST_ERR_LABEL_RANGE);
    int total;
    (void)block_rank(valid, wave_total, total);
    if (threadIdx.x == 0) block_cnt[blockIdx.x] = total;
}

// One workgroup: block_ofs[b] = sum of block_cnt[0 .. b), M and g/M into the header.
__global__ __launch_bounds__(kScanThreads) void block_offsets_kernel(
    const int32_t* __restrict__ block_cnt, int64_t nblocks, int64_t* __restrict__ block_ofs,
    Header* h, float grad_loss, int sum_mode, int64_t* __restrict__ n_valid_out) {
    __shared__ long long part[kScanThreads];
    const int tid = threadIdx.x;
    // thread t owns the contiguous chunk [t * per, (t + 1) * per)
    const int64_t per = (nblocks + kScanThreads - 1) / kScanThreads;
    const int64_t lo = tid * per, hi = lo + per < nblocks ? lo + per : nblocks;
    long long sum = 0;
    for (int64_t b = lo; b < hi; ++b) sum += block_cnt[b];
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        long long run = 0;
        for (int t = 0; t < kScanThreads; ++t) {
            const long long c = part[t];
            part[t] = run;
            run += c;
        }
        h->n_valid = run;
        // gradient scale: g / M for the mean, g for the sum of the token losses
        h->inv = run > 0 ? (sum_mode ? grad_loss : grad_loss / (float)run) : 0.f;
        if (n_valid_out) *n_valid_out = run;
    }
    __syncthreads();
    long long run = part[tid];
    for (int64_t b = lo; b < hi; ++b) {
        block_ofs[b] = run;
        run += block_cnt[b];
    }
}

__global__ __launch_bounds__(kScanThreads) void scatter_index_kernel(
    const int32_t* __restrict__ labels, int64_t N, int H, int ignore_index, int V,
    const int64_t* __restrict__ block_ofs, int32_t* __restrict__ idx, float* __restrict__ lse,
    float* __restrict__ loss_rows, uint16_t* __restrict__ dHidden) {
    __shared__ int wave_total[kScanThreads / 64];
    __shared__ unsigned char is_valid[kScanThreads];
    const int64_t row0 = (int64_t)blockIdx.x * kScanThreads;
    const int64_t i = row0 + threadIdx.x;
    const int y = i < N ? labels[i] : ignore_index;
    const bool valid = i < N && label_valid(y, ignore_index, V);
    int total;
    const int rank = block_rank(valid, wave_total, total);
    is_valid[threadIdx.x] = valid ? 1 : 0;
    if (valid) idx[block_ofs[blockIdx.x] + rank] = (int32_t)i;
    else if (i < N) {
        if (lse) lse[i] = 0.f;
        if (loss_rows) loss_rows[i] = 0.f;
    }
    if (!dHidden || total == kScanThreads) return;
    __syncthreads();
    const int chunks = H / 8;
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};
    for (int r = 0; r < kScanThreads && row0 + r < N; ++r) {
        if (is_valid[r]) continue;
        u32x4_t* dst = reinterpret_cast<u32x4_t*>(dHidden + (row0 + r) * H);
        for (int c = threadIdx.x; c < chunks; c += kScanThreads) dst[c] = zero4;
    }
}

// The counts of tile t (dense rows [t T, t T + T) cut at M) and its k offset inside its dW group.
__global__ void tile_info_kernel(const Header* __restrict__ h, int64_t t, int64_t T,
                                 TileInfo* __restrict__ info, const TileInfo* __restrict__ prev,
                                 int64_t H, int64_t V, int64_t Tp, int64_t dh_patches,
                                 int64_t dh_part_rows, int PR, int PC) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    long long left = h->n_valid - t * T;
    const int Tc = (int)(left < 0 ? 0 : (left > T ? T : left));
    const int Trc = (Tc + kBlockR - 1) / kBlockR * kBlockR;
    info->Tc = Tc;
    info->Trc = Trc;
    info->Tkc = (Tc + kBlockK - 1) / kBlockK * kBlockK;
    info->kofs = prev ? prev->kofs + prev->Tkc : 0;     // prev: the tile before, same dW group
    // dHidden of this tile: as many ranges of V as fill the chip best for its Trc rows, within
    // what the launch and the buffer of partial products were sized for
    int sp = 1, ks = (int)((V + kBlockK - 1) / kBlockK);
    if (Trc > 0) {
        dhidden_splits(Trc, H, V, dh_part_rows, sp, ks);
        const PatchGrid g = {Trc / kBlockR, (int)((H + kBlockC - 1) / kBlockC), PR, PC};
        if ((int64_t)g.patches() * sp > dh_patches || (sp > 1 && (int64_t)sp * Trc > dh_part_rows))
            dhidden_splits(Tp, H, V, 0, sp, ks);        // the full tile's choice always fits
        if ((int64_t)g.patches() * sp > dh_patches || (sp > 1 && (int64_t)sp * Trc > dh_part_rows)) {
            sp = 1;
            ks = (int)((V + kBlockK - 1) / kBlockK);
        }
    }
    info->splits = sp;
    info->ksteps = ks;
    info->redo = 0;
}

// Block b: dense row b of the tile.  Copies the hidden row of token idx_t[b] into the dense
// matrix Hc (row pitch Hk = H rounded up to whole k-steps, zeros behind the H elements: the logits
// GEMM contracts over Hk) and its label into yc; rows Tc <= b < Trc are zero padding.  Hc holds
// the whole dW group and the tile's rows start at its k offset.  Also sets the row's softmax reference for the
// first logits pass (0; backward from a saved lse: that lse, so that e is the probability itself)
// and marks the row as taking part in that pass.
__global__ __launch_bounds__(256) void gather_rows_kernel(
    const uint16_t* __restrict__ hidden, const int32_t* __restrict__ labels, int H, int Hk,
    const int32_t* __restrict__ idx_t, const TileInfo* __restrict__ info,
    const float* __restrict__ lse_in, uint16_t* __restrict__ Hc, int32_t* __restrict__ yc,
    float* __restrict__ ref, int32_t* __restrict__ rowstate) {
    const int b = blockIdx.x;
    const int chunks = Hk / 8, src_chunks = H / 8;      // the row pitch Hk is H in whole k-steps
    if (b >= info->Trc) return;
    Hc += (int64_t)info->kofs * Hk;
    u32x4_t* dst = reinterpret_cast<u32x4_t*>(Hc + (int64_t)b * Hk);
    if (b < info->Tc) {
        const int64_t row = idx_t[b];
        const u32x4_t* src = reinterpret_cast<const u32x4_t*>(hidden + row * H);
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        for (int c = threadIdx.x; c < chunks; c += 256) dst[c] = c < src_chunks ? src[c] : zero4;
        if (threadIdx.x == 0) {
            yc[b] = labels[row];
            ref[b] = lse_in ? lse_in[row] : 0.f;
            rowstate[b] = 1;
        }
    } else {
        const u32x4_t zero4 = {0u, 0u, 0u, 0u};
        for (int c = threadIdx.x; c < chunks; c += 256) dst[c] = zero4;
        if (threadIdx.x == 0) {
            yc[b] = -1;
            ref[b] = 0.f;
            rowstate[b] = 1;
        }
    }
}

enum { MODE_FWD = 0, MODE_FUSED = 1, MODE_BWD = 2 };

// A row's e = exp(z - ref) live in bf16 (the stash) and in fp32 sums; both have 8 exponent bits.
// With S = sum_v e inside [kSumLo, kSumHi] no e of weight overflows, the ones that underflow are
// below 2^-66 of the row's mass, and the fp32 products S * |w| of the dHidden contraction stay far
// from overflow.  A row outside is redone with ref = its exact maximum (then 1 <= S <= V).
constexpr float kSumLo = 8.673617379884035e-19f;      // 2^-60
constexpr float kSumHi = 1.2676506002282294e30f;      // 2^100
constexpr float kLog2e = 1.4426950408889634f;

struct RowFinishParams {
    const float* pm;         // [ng, Tp]  per 128-column group: max z          (first pass only)
    const float* ps;         // [ng, Tp]  per 128-column group: sum of e
    const float* zlabel;     // [Tp]      label logit of each dense row
    const int32_t* yc;       // [Tp]      label of each dense row
    const int32_t* idx;      // [Tp]      dense row -> row of the sequence
    TileInfo* info;
    float* ref;              // [Tp]      the row's reference; rewritten for a row that is redone
    float* frow;             // [Tp]      1 / S of a finished row (MODE_FUSED), 1 (MODE_BWD)
    int32_t* rowstate;       // [Tp]      1: the row takes part in the next logits pass, 0: finished
    float* lse_t;            // [N]       by row of the sequence
    float* loss_rows_t;      // [N]
    uint16_t* hc;            // [Kg, Hk]  dense hidden rows of the group (scaled in place, MODE_FUSED)
    uint16_t* stash;         // [Kg, Vp]
    int Tp, ng, H, Hk, Vp;
};

// Per dense row of the tile, after a logits pass: S = sum of the per-group sums of e (fixed order,
// so a row's lse depends on nothing but its own partials), lse = ref + log S, the row's loss term
// (both written to the row's original position) and, when gradients follow,
//   * the stash entry of the label becomes e_label - S (MODE_FUSED) or p_label - 1 (MODE_BWD),
//     formed in fp32 from the label logit, so that (stash * f)[v] = p[v] - [v = label] with the
//     relative precision of bf16 in every entry;
//   * frow = f = 1 / S (adjusted by the rounding of the label entry, see below), which dHidden
//     applies to its output rows;
//   * the row's dense hidden row is multiplied by f in place: it is the other operand of the
//     dW product, whose contraction index is the row.
// First pass (REDO = false): a row whose S is outside [kSumLo, kSumHi] is not finished; its
// reference becomes its exact maximum, it stays marked, and the tile is flagged for the second
// pass.  Second pass (REDO = true): leaves at once unless flagged; finishes the marked rows.
// MODE_BWD has no sums to combine (e is the probability itself): label entries only.
// Block = 16 rows x 64 lanes: thread (x, y) owns groups y, y + 64, ... of row x; the 64 lanes of a
// row are combined through LDS in a fixed order.
constexpr int kCombineRows = 16, kCombineLanes = 64;
template <int MODE, bool REDO>
__global__ __launch_bounds__(kCombineRows * kCombineLanes) void row_finish_kernel(const RowFinishParams p) {
    __shared__ float red[kCombineLanes][kCombineRows];
    const int x = threadIdx.x, y = threadIdx.y;
    if ((int)blockIdx.x * kCombineRows >= p.info->Trc) return;
    if (REDO && !p.info->redo) return;
    const int i = blockIdx.x * kCombineRows + x;          // dense row; Trc is a multiple of 256
    const bool inrow = i < p.info->Tc;                    // every dense row below Tc is valid
    const bool marked = p.rowstate[i] != 0;
    __syncthreads();                                      // every thread of a row has read its mark
    const int Tp = p.Tp, ng = p.ng;
    float S = 1.f, M = 0.f;
    if (MODE != MODE_BWD) {
        float sum = 0.f;
        for (int g = y; g < ng; g += kCombineLanes) sum += p.ps[(int64_t)g * Tp + i];
        red[y][x] = sum;
        __syncthreads();
        S = red[0][x];
#pragma unroll
        for (int l = 1; l < kCombineLanes; ++l) S += red[l][x];
        __syncthreads();
        if (!REDO) {
            float m = -INFINITY;
            for (int g = y; g < ng; g += kCombineLanes) m = fmaxf(m, p.pm[(int64_t)g * Tp + i]);
            red[y][x] = m;
            __syncthreads();
            M = red[0][x];
#pragma unroll
            for (int l = 1; l < kCombineLanes; ++l) M = fmaxf(M, red[l][x]);
        }
    }
    // (rowstate, ref and frow of row i are written by the row's thread y == 0 only, and read above
    // or below by the same thread or before the barriers)
    if (!inrow) {                                         // padding rows: nothing to finish
        if (y == 0 && !REDO) { p.rowstate[i] = 0; p.frow[i] = 0.f; }
        return;
    }
    if (!marked) return;
    const bool ok = MODE == MODE_BWD || REDO || (S >= kSumLo && S <= kSumHi);
    if (!ok) {
        if (y == 0) {
            p.ref[i] = (M == -INFINITY || M != M) ? 0.f : M;
            atomicOr(&p.info->redo, 1);
        }
        return;
    }
    const int kofs = p.info->kofs;
    const float ref = p.ref[i], zl = p.zlabel[i];
    // the label's e, as the logits pass formed it before rounding it to bf16, minus S (MODE_BWD:
    // p - 1, S = 1), rounded to bf16 for the stash
    const float el = __builtin_amdgcn_exp2f(fmaf(zl, kLog2e, -(ref * kLog2e)));
    const __bf16 d = (__bf16)(el - S);
    // The row's scale is chosen so that the ROUNDED label entry times the scale is p - 1 to fp32
    // precision (the label entries carry the largest gradients); every other entry of the row then
    // sees the scale off by the label entry's rounding, within the 2^-9 its own rounding has.
    float f = 1.f / S;
    if (MODE != MODE_FWD && (float)d != 0.f) f = ((el - S) / (float)d) / S;     // (d * S may overflow)
    if (y == 0) {
        if (MODE != MODE_BWD) {
            const int orig = p.idx[i];
            const float lse = ref + __logf(S);
            p.lse_t[orig] = lse;
            p.loss_rows_t[orig] = lse - zl;
        }
        if (MODE != MODE_FWD) {
            p.stash[(int64_t)(kofs + i) * p.Vp + p.yc[i]] = __builtin_bit_cast(uint16_t, d);
            p.frow[i] = f;
        }
        p.rowstate[i] = 0;
    }
    if (MODE == MODE_FUSED) {
        uint16_t* row = p.hc + (int64_t)(kofs + i) * p.Hk;
        for (int c = y; c < p.H / 8; c += kCombineLanes) {
            bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(row + c * 8);
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = (__bf16)((float)v[q] * f);
            *reinterpret_cast<bf16x8_t*>(row + c * 8) = v;
        }
    }
}

// loss = (sum of the per-row terms in a fixed order) / M, or the sum itself.  One block.
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ loss_rows,
                                                           int64_t N, Header* h, int sum_mode,
                                                           float* __restrict__ loss_out) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < N; i += 1024) s += (double)loss_rows[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const long long M = h->n_valid;
        const double L = M > 0 ? (sum_mode ? part[0] : part[0] / (double)M) : 0.0;
        h->loss_sum = part[0];
        *loss_out = (float)L;
        if (!isfinite(L)) atomicMax(&h->status, (int)ALST_ERR_NONFINITE);
    }
}

// dW = (g/M) acc  (bf16 or fp32, overwrite or +=).  acc may alias dW (fp32 overwrite mode).
template <bool OUT_F32, bool ACCUM>
__global__ void dw_finalize_kernel(const float* acc, void* dW, int64_t n4, const Header* h) {
    const float inv = h->inv;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
         i += (int64_t)gridDim.x * blockDim.x) {
        f32x4_t a = reinterpret_cast<const f32x4_t*>(acc)[i];
        a *= inv;
        if (OUT_F32) {
            f32x4_t* o = reinterpret_cast<f32x4_t*>(dW) + i;
            if (ACCUM) a += *o;
            *o = a;
        } else {
            bf16x4_t* o = reinterpret_cast<bf16x4_t*>(dW) + i;
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

__global__ void copy_f32_kernel(const float* __restrict__ in, float* __restrict__ out, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        out[i] = in[i];
}

__global__ void shift_labels_kernel(const int32_t* __restrict__ labels, int32_t* __restrict__ out,
                                    int64_t N, int ignore_index) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x)
        out[i] = i + 1 < N ? labels[i + 1] : ignore_index;
}

// ---------------------------------------------------------------------------------------------
// the three block GEMMs
// ---------------------------------------------------------------------------------------------
struct LogitsParams {
    const uint16_t* hidden_t;   // [Kg, Hk]     dense (valid) rows of the dW group; the tile's rows
                                //              start at its k offset and are zero padded to Trc
    const uint16_t* W;          // [V, H]
    const int32_t* labels_t;    // [Tp]         labels of the dense rows
    const TileInfo* info;
    const float* ref;           // [Tp]         reference of each dense row: e = exp(z - ref)
    const int32_t* rowstate;    // [Tp]         second pass: rows that are redone (others keep their results)
    float* pm;                  // [ng, Tp]     MODE_FWD / MODE_FUSED
    float* ps;                  // [ng, Tp]
    float* zlabel;              // [Tp]
    uint16_t* stash;            // [Kg, Vp]     MODE_FUSED / MODE_BWD; rows as in hidden_t
    int Tp, H, Hk, V, Vp;       // Tp = row stride of the per-tile arrays
    int PR, PC;                 // patch shape of the block -> tile mapping
};

// r = token row of the tile (MFMA lane dimension), c = vocabulary id (register dimension).
// KTAIL: the hidden size is not whole k-steps; the contraction runs over Hk, the dense hidden rows
// are zero beyond H and the chunks of W's rows beyond H are read from each row's last chunk.
// REDO: the second pass over a tile, for the rows whose first-pass sums left the safe range; its
// workgroups leave at once unless row_finish flagged the tile, and rows that are not marked keep
// what the first pass wrote.
template <class Core, bool KTAIL, int MODE, bool REDO>
__global__ __launch_bounds__(Core::kThreads) void logits_kernel(const LogitsParams p) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    extern __shared__ __align__(16) unsigned char smem[];
    int tr, tc;
    const int T_cur = p.info->Tc, Trc = p.info->Trc;
    if (T_cur == 0) return;
    if (REDO && !p.info->redo) return;
    {
        const PatchGrid pg = {Trc / kBlockR, p.Vp / kBlockC, p.PR, p.PC};
        int P, w;
        patch_of_block(blockIdx.x, P, w);
        if (P >= pg.patches() || !tile_in_patch(pg, P, w, tr, tc)) return;
    }
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;
    constexpr int kRegs = 4 * Core::kRuns;          // accumulator registers of a tile

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    const int kofs = p.info->kofs;
    const uint16_t* const hidden_t = p.hidden_t + (int64_t)kofs * p.Hk;
    const uint16_t* warm = warm_row(p.PR, p.PC, hidden_t, p.Hk, r0, tr, p.W, p.H, c0, tc, nullptr, p.V);
    Core::template gemm<false, KTAIL>(hidden_t, p.Hk, Trc, p.W, p.H, p.V, p.Hk, r0, c0, smem, acc, warm,
                                      kBlockK, nullptr, p.H);

    const typename Core::Lane lp;
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) {
        const int i = r0 + lp.r(nt);
        const bool rowok = i < T_cur;
        const bool act = !REDO || p.rowstate[i] != 0;     // this pass writes row i's results
        {                               // columns beyond the vocabulary (last column block)
            if (c0 + kBlockC > p.V) {
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int j = 0; j < kRegs; ++j)
                        if (c0 + lp.c(mt, j >> 2) + (j & 3) >= p.V) acc[mt][nt][j] = -INFINITY;
            }
        }
        const float ref = p.ref[i];
        float m = 0.f;
        if (MODE != MODE_BWD && !REDO) {                  // the row's exact maximum, for a redo
            m = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                for (int j = 0; j < kRegs; ++j) m = fmaxf(m, acc[mt][nt][j]);
            m = groups_max<Core::kGroups>(m);
        }
        {
            // label logit: exactly one lane of one block holds column y of row i.  Few wavefronts
            // hold any (a tile's rows x 128 of V columns), so the search sits behind a uniform branch.
            const int y = rowok && act ? p.labels_t[i] : -1;
            const unsigned d = (unsigned)(y - (c0 + lp.wc * kGroupC));
            const bool mine = y >= 0 && d < (unsigned)kGroupC &&
                              ((d >> 2) & (unsigned)(Core::kGroups - 1)) == (unsigned)lp.grp;
            if (__ballot(mine) != 0ull) {
                if (mine) {
                    float zl = 0.f;
#pragma unroll
                    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                        for (int j = 0; j < kRegs; ++j)
                            if (d == (unsigned)(lp.cw(mt, j >> 2) + (j & 3))) zl = acc[mt][nt][j];
                    p.zlabel[i] = zl;
                }
            }
        }
        // e = exp(z - ref) as exp2(z * log2(e) - ref * log2(e)); summed in fp32, stored as bf16.
        // In the accumulators a lane holds 4 consecutive columns of one row, so a direct store
        // would scatter 8-byte pieces over many rows per instruction.  The wavefront instead turns
        // its kTile x 128 piece around in LDS (free once the k-loop is over; each wavefront has its
        // own region and LDS serves a wavefront's accesses in order, so no barrier is needed) and
        // stores whole 256-byte row segments.
        const float ref2 = ref * kLog2e;
        unsigned char* const tw = smem + (threadIdx.x >> 6) * (32 * kTurnPitch);
        float s = 0.f;
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int q = 0; q < Core::kRuns; ++q) {
                bf16x4_t o;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float e = __builtin_amdgcn_exp2f(fmaf(acc[mt][nt][q * 4 + x], kLog2e, -ref2));
                    s += e;
                    o[x] = (__bf16)e;
                }
                if (MODE != MODE_FWD)
                    *reinterpret_cast<bf16x4_t*>(tw + lp.lrow * kTurnPitch + lp.cw(mt, q) * 2) = o;
            }
        if (MODE != MODE_FWD) {
            const int lrow = lp.lane >> 4, lcol = lp.lane & 15;        // 4 rows x 16 chunks of 16 B
            const int rb = r0 + lp.rbase(nt);
            uint16_t* const out = p.stash + (int64_t)(kofs + rb) * p.Vp + c0 + lp.wc * kGroupC + lcol * 8;
#pragma unroll
            for (int it = 0; it < Core::kTile / 4; ++it) {
                const int row = it * 4 + lrow;
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(tw + row * kTurnPitch + lcol * 16);
                if (!REDO || p.rowstate[rb + row] != 0)
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(out + (int64_t)row * p.Vp));
            }
        }
        if (MODE != MODE_BWD) {
            s = groups_sum<Core::kGroups>(s);
            if (lp.grp == 0 && act) {
                const int64_t g = (c0 + lp.wc * kGroupC) >> 7;
                if (!REDO) p.pm[g * p.Tp + i] = m;
                p.ps[g * p.Tp + i] = s;
            }
        }
    }
}

struct DHiddenParams {
    const uint16_t* dz;      // [Kg, Vp]     dense rows of the dW group; the tile starts at its k offset
    const uint16_t* Wt;      // [H, Vp]      W transposed (k = vocabulary id contiguous), zero beyond V
    uint16_t* dH_t;          // [N, H]       whole dHidden; dense row i goes to row idx[i]
    const int32_t* idx;
    const TileInfo* info;
    const Header* hdr;
    const float* frow;       // [Tp]         scale of each dense row's result: 1 / S of its softmax
    float* part;             // [splits, Trc, H] fp32 partial products (splits > 1); the number
                             // of ranges and their length are the tile's (TileInfo)
    int Tp, H, V, Vp;
    int PR, PC;              // patch shape of the block -> tile mapping
};

// dH = dZ W runs with both operands k-contiguous (the fastest of the block GEMM's layouts: 9 % on
// this product): W transposed, [H, Vp] with zeros for V <= v < Vp, is made once per call that
// computes gradients (transpose_bf16_kernel), for the price of reading and writing W once.

// r = token row (lane dimension), c = hidden index (register dimension), k = vocabulary; both
// operands k-contiguous (dZ rows and the rows of W transposed).
// The output has only (T / 256) * (H / 256) blocks, each with a long contraction: when that
// number does not fill the compute units evenly, the contraction is cut into `splits` ranges, each
// range's blocks write fp32 partial products, and dhidden_reduce_kernel adds them in a fixed
// order.
template <class Core>
__global__ __launch_bounds__(Core::kThreads) void dhidden_kernel(const DHiddenParams p) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    extern __shared__ __align__(16) unsigned char smem[];
    int tr, tc;
    const int tiles_c = (p.H + kBlockC - 1) / kBlockC;
    const int T_cur = p.info->Tc, Trc = p.info->Trc;
    if (T_cur == 0) return;
    // the ranges are parts of one launch: their patches are numbered through
    const PatchGrid pg = {Trc / kBlockR, tiles_c, p.PR, p.PC};
    int P, w;
    patch_of_block(blockIdx.x, P, w);
    const int np = pg.patches(), split = P / np;
    const int splits = p.info->splits, ksteps = p.info->ksteps;
    if (split >= splits || !tile_in_patch(pg, P - split * np, w, tr, tc)) return;
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;
    // k runs over V rounded up to whole k-steps: dZ and Wt are zero there
    const int k0 = split * ksteps * kBlockK;
    const int klen = min(ksteps * kBlockK, (p.V + kBlockK - 1) / kBlockK * kBlockK - k0);     // > 0

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    const uint16_t* const dz = p.dz + (int64_t)p.info->kofs * p.Vp + k0;
    const uint16_t* const Wk = p.Wt + k0;
    // (a hidden size that ends inside the block: the rows of Wt beyond H are read from its last
    // row, and the epilogue skips those columns)
    const uint16_t* warm = warm_row(p.PR, p.PC, dz, p.Vp, r0, tr, Wk, p.Vp, c0, tc, nullptr, p.H);
    Core::template gemm<false>(dz, p.Vp, Trc, Wk, p.Vp, p.H, klen, r0, c0, smem, acc, warm);

    const typename Core::Lane lp;
    if (splits > 1) {
        float* const part = p.part + (int64_t)split * Trc * p.H;
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt) {
            float* row = part + (int64_t)(r0 + lp.r(nt)) * p.H;
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                for (int q = 0; q < Core::kRuns; ++q) {
                    const int h = c0 + lp.c(mt, q);
                    if (h >= p.H) continue;             // last column block of a ragged H
                    f32x4_t o;
#pragma unroll
                    for (int x = 0; x < 4; ++x) o[x] = acc[mt][nt][q * 4 + x];
                    *reinterpret_cast<f32x4_t*>(row + h) = o;
                }
        }
        return;
    }
    const float inv = p.hdr->inv;
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) {
        const int i = r0 + lp.r(nt);
        if (i >= T_cur) continue;
        const float sc = inv * p.frow[i];
        uint16_t* row = p.dH_t + (int64_t)p.idx[i] * p.H;
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int q = 0; q < Core::kRuns; ++q) {
                const int h = c0 + lp.c(mt, q);
                if (h >= p.H) continue;             // last column block of a ragged H
                bf16x4_t o;
#pragma unroll
                for (int x = 0; x < 4; ++x) o[x] = (__bf16)(acc[mt][nt][q * 4 + x] * sc);
                *reinterpret_cast<bf16x4_t*>(row + h) = o;
            }
    }
}

// dH[idx[i]] = (g/M) (1/S_i) * sum over the ranges of the partial products of dense row i, in
// range order.  Tiles whose contraction was not cut were written by dhidden_kernel itself.
__global__ __launch_bounds__(256) void dhidden_reduce_kernel(const float* __restrict__ part, int H,
                                                             const int32_t* __restrict__ idx,
                                                             const TileInfo* __restrict__ info,
                                                             const Header* __restrict__ hdr,
                                                             const float* __restrict__ frow,
                                                             uint16_t* __restrict__ dH) {
    const int i = blockIdx.x;
    const int splits = info->splits, Trc = info->Trc;
    if (i >= info->Tc || splits <= 1) return;
    const float inv = hdr->inv * frow[i];
    uint16_t* out = dH + (int64_t)idx[i] * H;
    for (int c = threadIdx.x * 4; c < H; c += 256 * 4) {
        f32x4_t a = *reinterpret_cast<const f32x4_t*>(part + (int64_t)i * H + c);
        for (int sp = 1; sp < splits; ++sp)
            a += *reinterpret_cast<const f32x4_t*>(part + ((int64_t)sp * Trc + i) * H + c);
        bf16x4_t o;
#pragma unroll
        for (int x = 0; x < 4; ++x) o[x] = (__bf16)(a[x] * inv);
        *reinterpret_cast<bf16x4_t*>(out + c) = o;
    }
}

struct DWParams {
    const uint16_t* hg;      // [Kg, Hk]     dense hidden rows of the group's tiles (H of the Hk columns used)
    const uint16_t* dzg;     // [Kg, Vp]     their dZ rows
    float* acc;              // [V, H]
    const TileInfo* info;    // of the group's last tile: k extent = kofs + Tkc
    int H, Hk, V, Vp;
    int first;               // first group: store instead of add
    int PR, PC;              // patch shape of the block -> tile mapping
};

// r = hidden index (lane dimension), c = vocabulary id (register dimension), k = dense token row:
// both operands have k as the slow index (k-major cores).  With the hidden index along the lanes
// the accumulate moves full 128-byte lines of acc (accumulate_block_f32).
template <class Core, bool GUARD>
__global__ __launch_bounds__(Core::kThreads) void dw_kernel(const DWParams p) {
    constexpr int kMT = Core::kMT, kNT = Core::kNT;
    extern __shared__ __align__(16) unsigned char smem[];
    int tr, tc;
    const int tiles_r = (p.H + kBlockR - 1) / kBlockR;
    const int Tkc = p.info->kofs + p.info->Tkc;      // k extent of the whole group
    if (Tkc == 0 && !p.first) return;
    {
        const PatchGrid pg = {tiles_r, p.Vp / kBlockC, p.PR, p.PC};
        int P, w;
        patch_of_block(blockIdx.x, P, w);
        if (P >= pg.patches() || !tile_in_patch(pg, P, w, tr, tc)) return;
    }
    const int r0 = tr * kBlockR, c0 = tc * kBlockC;

    typename Core::acc_t acc[kMT][kNT];
    zero_acc<Core>(acc);

    if (Tkc > 0) {
        int64_t step = 0;
        const uint16_t* warm = Core::kCanGuard ? nullptr
                                               : warm_line_kmajor(p.PR, p.PC, p.hg, p.Hk, r0, tr, p.dzg,
                                                                  p.Vp, c0, tc, step, p.H, p.Vp);
        Core::template gemm<GUARD>(p.hg, p.Hk, p.H, p.dzg, p.Vp, p.Vp, Tkc, r0, c0, smem, acc, warm, step);
    }

    accumulate_block_f32<Core, GUARD>(acc, p.acc, p.H, r0, c0, p.H, p.V, p.first != 0);
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static int prepare_kernels_on_current_device() {
    int rc = ALST_OK;
    auto acc = [&](int r) { if (r != ALST_OK) rc = r; };
    acc(allow_big_lds(logits_kernel<DirectCore, false, MODE_FWD, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, true, MODE_FWD, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, false, MODE_FUSED, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, true, MODE_FUSED, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, false, MODE_BWD, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, true, MODE_BWD, false>));
    acc(allow_big_lds(logits_kernel<DirectCore, false, MODE_FWD, true>));
    acc(allow_big_lds(logits_kernel<DirectCore, true, MODE_FWD, true>));
    acc(allow_big_lds(logits_kernel<DirectCore, false, MODE_FUSED, true>));
    acc(allow_big_lds(logits_kernel<DirectCore, true, MODE_FUSED, true>));
    acc(allow_big_lds(dhidden_kernel<DirectCore>));
    acc(allow_big_lds(dw_kernel<KMajorCore, false>));
    return rc;
}
// Once per device, whatever the number of host threads that make their first call together.
static int prepare_kernels() {
    static std::once_flag once[kMaxDevices];
    static int results[kMaxDevices];
    const int dev = current_device_slot();
    if (dev < 0) return ALST_ERR_HIP;
    std::call_once(once[dev], [dev] { results[dev] = prepare_kernels_on_current_device(); });
    return results[dev];
}

struct Problem {
    const uint16_t* hidden;
    const uint16_t* W;
    const int32_t* labels;
    const float* lse_in;
    int64_t N, H, V, tile;
    int ignore_index;
    float grad_loss;
    float* loss_out;
    float* lse_out;
    int64_t* n_valid_out;
    uint16_t* dHidden;
    void* dW;
    unsigned char* ws;
    uint32_t flags;
    hipStream_t stream;
};

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// own_scratch: the workspace is the library's own static buffer of workspace_bytes (P.ws is not
// looked at).
static int validate(const Problem& P, size_t workspace_bytes, bool need_fwd_out, bool need_bwd_out,
                    bool need_lse_in, bool own_scratch = false) {
    if (!P.hidden || !P.W || !P.labels || (!own_scratch && !P.ws)) return ALST_ERR_NULL;
    if (need_fwd_out && !P.loss_out) return ALST_ERR_NULL;
    if (need_bwd_out && (!P.dHidden || !P.dW)) return ALST_ERR_NULL;
    if (need_lse_in && !P.lse_in) return ALST_ERR_NULL;
    if (P.flags & ~kKnownFlags) return ALST_ERR_UNSUPPORTED;
    if (need_bwd_out && (P.flags & ALST_FLAG_FORWARD_ONLY)) return ALST_ERR_UNSUPPORTED;
    if (P.N < 1 || P.H < 1 || P.V < 1 || P.tile < 1) return ALST_ERR_SHAPE;
    if (P.N > (int64_t)1 << 30 || P.H > (int64_t)1 << 20 || P.V > (int64_t)1 << 24)
        return ALST_ERR_SHAPE;
    if (P.H % 8 != 0) return ALST_ERR_ALIGN;
    if (!aligned16(P.hidden) || !aligned16(P.W) || (!own_scratch && !aligned16(P.ws)))
        return ALST_ERR_ALIGN;
    if (need_bwd_out && (!aligned16(P.dHidden) || !aligned16(P.dW))) return ALST_ERR_ALIGN;
    const Layout L = make_layout(P.N, P.H, P.V, P.tile, P.flags);
    // every launch must fit a one-dimensional grid
    if (!checked_grid(L.Tp / kBlockR, L.Vp / kBlockC) ||
        !checked_grid((P.H + kBlockR - 1) / kBlockR, L.Vp / kBlockC) ||
        L.dh_patches * 32 > 0x7fffff00 ||                                        // dHidden
        (L.Vp / 256) * (L.Tp / 64) > 0x7fffffff)
        return ALST_ERR_SHAPE;
    if (workspace_bytes < L.total) return own_scratch ? ALST_ERR_NOALLOC_LIMIT : ALST_ERR_WORKSPACE;
    return ALST_OK;
}

// Grids are sized for Tr (the tile's rows rounded up to the block height); the kernels read the
// number of rows that take part from the device and surplus blocks leave at once.
template <int MODE, bool REDO>
static int launch_logits(LogitsParams lp, int Tr, bool ktail, hipStream_t s) {
    const PatchGrid pg = choose_patches(Tr / kBlockR, lp.Vp / kBlockC);
    lp.PR = pg.PR; lp.PC = pg.PC;
    const int grid = grid_for_patches(pg.patches());
    if (ktail)
        hipLaunchKernelGGL((logits_kernel<DirectCore, true, MODE, REDO>), dim3(grid),
                           dim3(DirectCore::kThreads), kLdsBytes, s, lp);
    else
        hipLaunchKernelGGL((logits_kernel<DirectCore, false, MODE, REDO>), dim3(grid),
                           dim3(DirectCore::kThreads), kLdsBytes, s, lp);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

// The logits pass of a tile and the per-row work behind it; for the modes that form the softmax
// sums, followed by the conditional second pass (see row_finish_kernel).
template <int MODE>
static int logits_and_finish(const LogitsParams& lp, const RowFinishParams& fp, int Tr, bool ktail,
                             hipStream_t s) {
    const dim3 fgrid(Tr / kCombineRows), fblock(kCombineRows, kCombineLanes);
    int rc;
    {
        ProfScope ps_(PROF_LOGITS, s);
        rc = launch_logits<MODE, false>(lp, Tr, ktail, s);
    }
    if (rc != ALST_OK) return rc;
    {
        ProfScope small_(PROF_OTHER, s);
        hipLaunchKernelGGL((row_finish_kernel<MODE, false>), fgrid, fblock, 0, s, fp);
        ALST_HIP(hipGetLastError());
    }
    if (MODE == MODE_BWD) return ALST_OK;
    constexpr int M2 = MODE == MODE_BWD ? MODE_FUSED : MODE;      // (MODE_BWD never gets here)
    // (timed with the small kernels: in all but pathological inputs both launches are empty)
    ProfScope small_(PROF_OTHER, s);
    rc = launch_logits<M2, true>(lp, Tr, ktail, s);
    if (rc != ALST_OK) return rc;
    hipLaunchKernelGGL((row_finish_kernel<M2, true>), fgrid, fblock, 0, s, fp);
    ALST_HIP(hipGetLastError());
    return ALST_OK;
}

// do_fwd: produce loss / lse.  do_bwd: produce gradients.  Both: one fused sweep.
static int run(const Problem& P, bool do_fwd, bool do_bwd) {
    int rc = prepare_kernels();
    if (rc != ALST_OK) return rc;
    const Layout L = make_layout(P.N, P.H, P.V, P.tile, P.flags);
    hipStream_t s = P.stream;
    Header* hdr = reinterpret_cast<Header*>(P.ws + L.header);
    TileInfo* infos = reinterpret_cast<TileInfo*>(P.ws + L.tinfo);
    float* loss_rows = reinterpret_cast<float*>(P.ws + L.loss_rows);
    float* lse_buf = P.lse_out ? P.lse_out : reinterpret_cast<float*>(P.ws + L.lse);
    float* zlabel = reinterpret_cast<float*>(P.ws + L.zlabel);
    int32_t* yc = reinterpret_cast<int32_t*>(P.ws + L.yc);
    int32_t* idx = reinterpret_cast<int32_t*>(P.ws + L.idx);
    int32_t* block_cnt = reinterpret_cast<int32_t*>(P.ws + L.block_cnt);
    int64_t* block_ofs = reinterpret_cast<int64_t*>(P.ws + L.block_ofs);
    float* pm = reinterpret_cast<float*>(P.ws + L.pm);
    float* ps = reinterpret_cast<float*>(P.ws + L.ps);
    float* ref = reinterpret_cast<float*>(P.ws + L.ref);
    float* frow = reinterpret_cast<float*>(P.ws + L.frow);
    int32_t* rowstate = reinterpret_cast<int32_t*>(P.ws + L.rowstate);
    uint16_t* hc = reinterpret_cast<uint16_t*>(P.ws + L.hc);
    uint16_t* stash = reinterpret_cast<uint16_t*>(P.ws + L.stash);
    uint16_t* wt = reinterpret_cast<uint16_t*>(P.ws + L.wt);
    const bool acc_in_dw = (P.flags & ALST_FLAG_DW_FP32) && !(P.flags & ALST_FLAG_DW_ACCUMULATE);
    float* acc = acc_in_dw ? reinterpret_cast<float*>(P.dW) : reinterpret_cast<float*>(P.ws + L.acc);

    const int H = (int)P.H, V = (int)P.V, Tp = (int)L.Tp, Vp = (int)L.Vp, ng = (int)L.ng;
    const int64_t T = P.tile < P.N ? P.tile : P.N;

    hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(64), 0, s, hdr);
    {
        const int64_t nblocks = (P.N + kScanThreads - 1) / kScanThreads;
        hipLaunchKernelGGL(block_count_kernel, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s,
                           P.labels, P.N, P.ignore_index, V, block_cnt, hdr);
        hipLaunchKernelGGL(block_offsets_kernel, dim3(1), dim3(kScanThreads), 0, s, block_cnt,
                           nblocks, block_ofs, hdr, P.grad_loss,
                           (P.flags & ALST_FLAG_REDUCE_SUM) ? 1 : 0, P.n_valid_out);
        hipLaunchKernelGGL(scatter_index_kernel, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s,
                           P.labels, P.N, H, P.ignore_index, V, block_ofs, idx,
                           do_fwd ? lse_buf : nullptr, do_fwd ? loss_rows : nullptr,
                           do_bwd ? P.dHidden : nullptr);
    }
    ALST_HIP(hipGetLastError());

    // The GEMM cores without bounds checks serve every shape.  The row extent of a tile is always
    // block-aligned (dense rows are zero padded to a multiple of the block height).
    // (a vocabulary that ends inside a column block: the logits kernel reads the last row of W
    // in place of the missing ones and masks those columns; a hidden size that is not whole
    // k-steps: the dense hidden rows are zero padded to Hk and the chunks of W's rows beyond H
    // are read from each row's last chunk)
    const bool ktail_logits = (H % kBlockK) != 0;
    // (a hidden size that ends inside a block is handled by the unguarded dHidden and dW kernels:
    // the missing rows of W transposed / columns of the dense hidden rows are read from the last
    // ones and the results discarded; a vocabulary that is not whole k-steps: dZ and W transposed
    // are zero up to the padded vocabulary)
    if (do_bwd) {
        ProfScope small_(PROF_OTHER, s);
        hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)(Vp / 64), (unsigned)((H + 63) / 64)), dim3(256),
                           0, s, reinterpret_cast<const uint16_t*>(P.W), V, H, (int64_t)H, wt, (int64_t)Vp);
        ALST_HIP(hipGetLastError());
    }

    // The host does not know M: it walks ceil(N / T) tiles, the most there can be; the kernels of
    // a tile beyond the dense rows find Tc = 0 on the device and leave at once.
    const int64_t ntiles = (P.N + T - 1) / T;
    for (int64_t t = 0; t < ntiles; ++t) {
        const int T_cur = (int)T;
        const int Tr = (T_cur + kBlockR - 1) / kBlockR * kBlockR;
        const int slot = (int)(t % L.g);                // position inside the dW group
        TileInfo* info = infos + slot;
        const int32_t* idx_t = idx + t * T;             // the tile's dense rows -> sequence rows

        {
            ProfScope small_(PROF_OTHER, s);
            hipLaunchKernelGGL(tile_info_kernel, dim3(1), dim3(64), 0, s, hdr, t, T, info,
                               slot ? info - 1 : nullptr, P.H, P.V, L.Tp, L.dh_patches, L.dh_part_rows,
                               L.dh_PR, L.dh_PC);
            hipLaunchKernelGGL(gather_rows_kernel, dim3(Tr), dim3(256), 0, s, P.hidden, P.labels, H,
                               (int)L.Hk, idx_t, info, do_fwd ? nullptr : P.lse_in, hc, yc, ref, rowstate);
            ALST_HIP(hipGetLastError());
        }

        LogitsParams lp;
        lp.hidden_t = hc;
        lp.W = P.W;
        lp.labels_t = yc;
        lp.info = info;
        lp.ref = ref; lp.rowstate = rowstate;
        lp.pm = pm; lp.ps = ps; lp.zlabel = zlabel; lp.stash = stash;
        lp.Tp = Tp; lp.H = H; lp.Hk = (int)L.Hk; lp.V = V; lp.Vp = Vp;
        RowFinishParams fp;
        fp.pm = pm; fp.ps = ps; fp.zlabel = zlabel; fp.yc = yc; fp.idx = idx_t; fp.info = info;
        fp.ref = ref; fp.frow = frow; fp.rowstate = rowstate;
        fp.lse_t = lse_buf; fp.loss_rows_t = loss_rows; fp.hc = hc; fp.stash = stash;
        fp.Tp = Tp; fp.ng = ng; fp.H = H; fp.Hk = (int)L.Hk; fp.Vp = Vp;
        if (do_fwd && do_bwd) rc = logits_and_finish<MODE_FUSED>(lp, fp, Tr, ktail_logits, s);
        else if (do_fwd) rc = logits_and_finish<MODE_FWD>(lp, fp, Tr, ktail_logits, s);
        else rc = logits_and_finish<MODE_BWD>(lp, fp, Tr, ktail_logits, s);
        if (rc != ALST_OK) return rc;
        if (!do_bwd) continue;

        {
            DHiddenParams dp;
            dp.dz = stash; dp.Wt = wt; dp.dH_t = P.dHidden; dp.idx = idx_t;
            dp.info = info; dp.hdr = hdr; dp.frow = frow;
            dp.part = reinterpret_cast<float*>(P.ws + L.part);
            dp.Tp = Tp; dp.H = H; dp.V = V; dp.Vp = Vp;
            dp.PR = L.dh_PR; dp.PC = L.dh_PC;
            // enough workgroups for whatever number of rows and ranges the tile turns out to have
            const int grid = grid_for_patches(L.dh_patches);
            ProfScope ps_(PROF_DHIDDEN, s);
            hipLaunchKernelGGL((dhidden_kernel<DirectCore>), dim3(grid), dim3(DirectCore::kThreads), kLdsBytes,
                               s, dp);
            if (L.dh_part_rows > 0)
                hipLaunchKernelGGL(dhidden_reduce_kernel, dim3(Tr), dim3(256), 0, s, dp.part, H, idx_t,
                                   info, hdr, frow, P.dHidden);
            ALST_HIP(hipGetLastError());
        }
        if (slot == L.g - 1 || t == ntiles - 1) {           // the group is complete
            DWParams wp;
            wp.hg = hc; wp.dzg = stash; wp.acc = acc; wp.info = info;
            wp.H = H; wp.Hk = (int)L.Hk; wp.V = V; wp.Vp = Vp; wp.first = (t < L.g);
            const PatchGrid pg = choose_patches((H + kBlockR - 1) / kBlockR, Vp / kBlockC);
            wp.PR = pg.PR; wp.PC = pg.PC;
            const int grid = grid_for_patches(pg.patches());
            ProfScope ps_(PROF_DW, s);
            hipLaunchKernelGGL((dw_kernel<KMajorCore, false>), dim3(grid), dim3(KMajorCore::kThreads),
                               kLdsBytes, s, wp);
            ALST_HIP(hipGetLastError());
        }
    }

    if (do_fwd) {
        hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, loss_rows, P.N, hdr,
                           (P.flags & ALST_FLAG_REDUCE_SUM) ? 1 : 0, P.loss_out);
        ALST_HIP(hipGetLastError());
    }
    if (do_bwd) {
        const int64_t n4 = P.V * P.H / 4;
        int blocks = (int)((n4 + 255) / 256);
        if (blocks > 8192) blocks = 8192;
        const bool f32 = P.flags & ALST_FLAG_DW_FP32, accum = P.flags & ALST_FLAG_DW_ACCUMULATE;
        if (f32 && accum)
            hipLaunchKernelGGL((dw_finalize_kernel<true, true>), dim3(blocks), dim3(256), 0, s, acc, P.dW, n4, hdr);
        else if (f32)
            hipLaunchKernelGGL((dw_finalize_kernel<true, false>), dim3(blocks), dim3(256), 0, s, acc, P.dW, n4, hdr);
        else if (accum)
            hipLaunchKernelGGL((dw_finalize_kernel<false, true>), dim3(blocks), dim3(256), 0, s, acc, P.dW, n4, hdr);
        else
            hipLaunchKernelGGL((dw_finalize_kernel<false, false>), dim3(blocks), dim3(256), 0, s, acc, P.dW, n4, hdr);
        ALST_HIP(hipGetLastError());
    }
    return ALST_OK;
}

// ---------------------------------------------------------------------------------------------
// the entry point that allocates nothing
// ---------------------------------------------------------------------------------------------
// The workspace of alst_tiled_ce_forward_backward_noalloc: one array per GPU, held from the moment
// the library's code is loaded on it until the process ends.  In host code the name `scratch` is
// only a handle for hipGetSymbolAddress; what the kernels get is the address that call returns
// for the current device (each GPU has its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[ALST_NOALLOC_SCRATCH_BYTES];

// The device address of `scratch` on the current device, looked up once per device.
static int noalloc_scratch(unsigned char** out) {
    static std::mutex lock;
    static unsigned char* ptrs[kMaxDevices];
    const int dev = current_device_slot();
    if (dev < 0) return ALST_ERR_HIP;
    std::lock_guard<std::mutex> hold(lock);
    if (!ptrs[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ALST_ERR_HIP;
        ptrs[dev] = static_cast<unsigned char*>(p);
    }
    *out = ptrs[dev];
    return ALST_OK;
}

__global__ void copy_status_kernel(const Header* __restrict__ h, int32_t* __restrict__ out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = h->status;
}

}  // namespace alst

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
using namespace alst;

extern "C" {

const char* alst_status_string(int status) {
    switch (status) {
        case ALST_OK: return "ok";
        case ALST_ERR_NULL: return "a required pointer is NULL";
        case ALST_ERR_SHAPE: return "N, H, V and tile must be >= 1 and within the supported range";
        case ALST_ERR_ALIGN: return "H must be a multiple of 8 and base pointers 16-byte aligned";
        case ALST_ERR_WORKSPACE: return "workspace is smaller than alst_tiled_ce_workspace_bytes()";
        case ALST_ERR_LABEL_RANGE: return "a label is neither ignore_index nor inside [0, V)";
        case ALST_ERR_HIP: return "a HIP runtime call or kernel launch failed";
        case ALST_ERR_UNSUPPORTED: return "unknown flag bits, or a flag this entry point does not take";
        case ALST_ERR_NONFINITE: return "the loss is not finite";
        case ALST_ERR_NOALLOC_LIMIT:
            return "the problem needs more scratch than the static buffer of "
                   "alst_tiled_ce_forward_backward_noalloc holds";
        default: return "unknown status";
    }
}

int alst_version(void) { return 100; }

size_t alst_tiled_ce_workspace_bytes(int64_t N, int64_t H, int64_t V, int64_t tile, uint32_t flags) {
    if (N < 1 || H < 1 || V < 1 || tile < 1) return 0;
    if (N > (int64_t)1 << 30 || H > (int64_t)1 << 20 || V > (int64_t)1 << 24) return 0;
    if (flags & ~kKnownFlags) return 0;
    return make_layout(N, H, V, tile, flags).total;
}

int alst_tiled_ce_forward(const void* hidden, const void* W, const int32_t* labels, int64_t N,
                          int64_t H, int64_t V, int64_t tile, int32_t ignore_index, float* loss_out,
                          float* lse_out, int64_t* n_valid_out, void* workspace,
                          size_t workspace_bytes, uint32_t flags, void* stream) {
    Problem P = {};
    P.hidden = (const uint16_t*)hidden; P.W = (const uint16_t*)W; P.labels = labels;
    P.N = N; P.H = H; P.V = V; P.tile = tile; P.ignore_index = ignore_index; P.grad_loss = 1.f;
    P.loss_out = loss_out; P.lse_out = lse_out; P.n_valid_out = n_valid_out;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate(P, workspace_bytes, true, false, false);
    if (rc != ALST_OK) return rc;
    return run(P, true, false);
}

int alst_tiled_ce_backward(const void* hidden, const void* W, const int32_t* labels,
                           const float* lse, int64_t N, int64_t H, int64_t V, int64_t tile,
                           int32_t ignore_index, float grad_loss, void* dHidden, void* dW,
                           void* workspace, size_t workspace_bytes, uint32_t flags, void* stream) {
    Problem P = {};
    P.hidden = (const uint16_t*)hidden; P.W = (const uint16_t*)W; P.labels = labels;
    P.lse_in = lse;
    P.N = N; P.H = H; P.V = V; P.tile = tile; P.ignore_index = ignore_index;
    P.grad_loss = grad_loss; P.dHidden = (uint16_t*)dHidden; P.dW = dW;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate(P, workspace_bytes, false, true, true);
    if (rc != ALST_OK) return rc;
    return run(P, false, true);
}

int alst_tiled_ce_forward_backward(const void* hidden, const void* W, const int32_t* labels,
                                   int64_t N, int64_t H, int64_t V, int64_t tile,
                                   int32_t ignore_index, float grad_loss, float* loss_out,
                                   float* lse_out, int64_t* n_valid_out, void* dHidden, void* dW,
                                   void* workspace, size_t workspace_bytes, uint32_t flags,
                                   void* stream) {
    Problem P = {};
    P.hidden = (const uint16_t*)hidden; P.W = (const uint16_t*)W; P.labels = labels;
    P.N = N; P.H = H; P.V = V; P.tile = tile; P.ignore_index = ignore_index;
    P.grad_loss = grad_loss; P.loss_out = loss_out; P.lse_out = lse_out;
    P.n_valid_out = n_valid_out; P.dHidden = (uint16_t*)dHidden; P.dW = dW;
    P.ws = (unsigned char*)workspace; P.flags = flags; P.stream = (hipStream_t)stream;
    const int rc = validate(P, workspace_bytes, true, true, false);
    if (rc != ALST_OK) return rc;
    return run(P, true, true);
}

int alst_tiled_ce_forward_backward_noalloc(const void* hidden, const void* W, const int32_t* labels,
                                           int64_t N, int64_t H, int64_t V, int64_t tile,
                                           int32_t ignore_index, float grad_loss, float* loss_out,
                                           float* lse_out, int64_t* n_valid_out, void* dHidden,
                                           void* dW, int32_t* device_status_out, uint32_t flags,
                                           void* stream) {
    Problem P = {};
    P.hidden = (const uint16_t*)hidden; P.W = (const uint16_t*)W; P.labels = labels;
    P.N = N; P.H = H; P.V = V; P.tile = tile; P.ignore_index = ignore_index;
    P.grad_loss = grad_loss; P.loss_out = loss_out; P.lse_out = lse_out;
    P.n_valid_out = n_valid_out; P.dHidden = (uint16_t*)dHidden; P.dW = dW;
    P.flags = flags; P.stream = (hipStream_t)stream;
    int rc = validate(P, ALST_NOALLOC_SCRATCH_BYTES, true, true, false, /*own_scratch=*/true);
    if (rc != ALST_OK) return rc;
    rc = noalloc_scratch(&P.ws);
    if (rc != ALST_OK) return rc;
    // run() starts by resetting the header and writes every other region of the workspace before
    // it reads it, so what the last call left in the array does not matter
    rc = run(P, true, true);
    if (rc != ALST_OK) return rc;
    if (device_status_out) {
        hipLaunchKernelGGL(copy_status_kernel, dim3(1), dim3(64), 0, P.stream,
                           reinterpret_cast<const Header*>(P.ws), device_status_out);
        if (hipGetLastError() != hipSuccess) return ALST_ERR_HIP;
    }
    return ALST_OK;
}

int alst_last_device_status(void* workspace, void* stream) {
    if (!workspace) return ALST_ERR_NULL;
    Header h;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ALST_ERR_HIP;
    if (hipMemcpy(&h, workspace, sizeof(Header), hipMemcpyDeviceToHost) != hipSuccess)
        return ALST_ERR_HIP;
    const int st = h.status;
    if (st != 0) {
        hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream,
                           reinterpret_cast<Header*>(workspace));
        if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ALST_ERR_HIP;
    }
    return st;
}

int alst_tiled_ce_token_losses(const void* workspace, size_t workspace_bytes, int64_t N, int64_t H,
                               int64_t V, int64_t tile, uint32_t flags, float* token_loss_out,
                               void* stream) {
    if (!workspace || !token_loss_out) return ALST_ERR_NULL;
    if (flags & ~kKnownFlags) return ALST_ERR_UNSUPPORTED;
    if (N < 1 || H < 1 || V < 1 || tile < 1) return ALST_ERR_SHAPE;
    if (N > (int64_t)1 << 30 || H > (int64_t)1 << 20 || V > (int64_t)1 << 24) return ALST_ERR_SHAPE;
    const Layout L = make_layout(N, H, V, tile, flags);
    if (workspace_bytes < L.total) return ALST_ERR_WORKSPACE;
    const float* rows = reinterpret_cast<const float*>((const unsigned char*)workspace + L.loss_rows);
    int blocks = (int)((N + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, rows,
                       token_loss_out, N);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

int alst_shift_labels(const int32_t* labels, int32_t* shift_labels, int64_t N, int32_t ignore_index,
                      void* stream) {
    if (!labels || !shift_labels) return ALST_ERR_NULL;
    if (N < 1 || N > (int64_t)1 << 30) return ALST_ERR_SHAPE;
    int blocks = (int)((N + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(shift_labels_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, labels,
                       shift_labels, N, ignore_index);
    return hipGetLastError() == hipSuccess ? ALST_OK : ALST_ERR_HIP;
}

}  // extern "C"
