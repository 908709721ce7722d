/*
 * alst.h -- C ABI of the MI355X (gfx950) sequence-tiled LM-head projection + cross-entropy.
 *
 * The operation (ALST paper, section "Sequence Tiling for Reducing Activation Memory
 * Footprint", the tiled logits + loss computation): the LM-head logits z = hidden * W^T are
 * never held for the whole sequence.  The sequence is cut into tiles of `tile` rows; for each
 * tile the logits are produced, consumed by the loss and by the gradients, and dropped, so the
 * memory the logits need is O(tile * V) instead of O(N * V).  Rows carry no cross-sequence
 * dependency, therefore the result equals the untiled projection + cross-entropy.
 * Labels (section "Loss Sharding in Hugging Face Transformers") are ALREADY shifted to line up
 * with the hidden rows; the library does no shifting.  A label equal to `ignore_index`
 * (-100 in the paper) leaves its token out of the loss.
 *
 *   z[i,v]  = sum_k hidden[i,k] W[v,k]            fp32 accumulation of bf16 products
 *   lse[i]  = log sum_v exp z[i,v]
 *   L       = (1/M) sum_{valid i} (lse[i] - z[i,label_i]),  M = #valid   (M == 0: L = 0, grads 0)
 *   dz[i,v] = (g/M) valid_i (exp(z[i,v]-lse[i]) - [v == label_i])
 *   dHidden = dz W          dW = dz^T hidden
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers unless the comment says host.  `stream` is a hipStream_t
 *     passed as void* (NULL = the default stream).
 *   - Layout: dense row-major, no strides: hidden[N,H], W[V,H], dHidden[N,H], dW[V,H].
 *     bf16 = bfloat16 (upper half of an IEEE binary32).  H must be a multiple of 8 and every
 *     base pointer 16-byte aligned, else ALST_ERR_ALIGN.  Any V >= 1 is accepted.  The fastest
 *     kernels are used for every V and every H that is a multiple of 64 (neither has to be a
 *     multiple of the 256-wide blocks the kernels work in); with another H the logits run on a
 *     slower, bounds-checked kernel.
 *   - Ownership: the caller owns every buffer, including `workspace`; the library allocates and
 *     frees no device memory and keeps no state between calls, so peak device memory is
 *     inputs + outputs + alst_tiled_ce_workspace_bytes().  Calls that share a workspace must be
 *     ordered on one stream; calls on different workspaces may come from different host threads.
 *     The one thing remembered is that a device's kernels have been given their LDS size
 *     attribute: the first compute call on each device sets it (once, behind a lock) and must
 *     therefore be made outside a HIP graph capture.
 *   - The functions validate on the host, enqueue work on `stream` and return without
 *     synchronising.  Outputs are valid once the stream has been synchronised.
 *   - Errors: an alst_status value is returned; host-detectable errors are returned before
 *     anything is enqueued.  Conditions only the device can see (a label that is neither
 *     ignore_index nor in [0,V), a non-finite loss) are recorded in a status word inside the
 *     workspace, read with alst_last_device_status().  A row with an out-of-range label is
 *     treated as ignored, so nothing is read or written out of bounds.
 *   - Rows of ignored tokens are left out of all three contractions: the rows with a valid label
 *     are numbered densely in sequence order and the tiles are cut from that dense numbering
 *     (tile t = valid rows t*tile .. t*tile+tile-1, gathered into a dense matrix), so the executed
 *     work is 6 * M * H * V flop for M valid tokens, not 6 * N * H * V.
 *   - tile: any value >= 1; a tile larger than N is clamped; N need not be a multiple of tile.
 *     The tile size changes scheduling and memory only: the loss bits do not depend on it.
 */
#ifndef ALST_H
#define ALST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ALST_OK = 0,
    ALST_ERR_NULL = 1,        /* a required pointer is NULL */
    ALST_ERR_SHAPE = 2,       /* N, H, V or tile < 1, or a size beyond the supported range */
    ALST_ERR_ALIGN = 3,       /* H % 8 != 0 or a base pointer not 16-byte aligned */
    ALST_ERR_WORKSPACE = 4,   /* workspace_bytes smaller than alst_tiled_ce_workspace_bytes() */
    ALST_ERR_LABEL_RANGE = 5, /* device: a label outside [0,V) that is not ignore_index */
    ALST_ERR_HIP = 6,         /* a HIP runtime call or kernel launch failed */
    ALST_ERR_UNSUPPORTED = 7, /* unknown flag bits, or a flag the entry point does not take */
    ALST_ERR_NONFINITE = 8,   /* device: the loss is not finite */
    ALST_ERR_NOALLOC_LIMIT = 9 /* alst_tiled_ce_forward_backward_noalloc: the problem needs more
                                 scratch than ALST_NOALLOC_SCRATCH_BYTES */
} alst_status;

/* dW is written as fp32 instead of bf16. */
#define ALST_FLAG_DW_FP32 1u
/* dW += gradient instead of dW = gradient (dHidden is always overwritten). */
#define ALST_FLAG_DW_ACCUMULATE 2u
/* The loss is the SUM of the token losses of the non-ignored tokens instead of their mean, and
 * the gradients are those of that sum (scaled by grad_loss instead of grad_loss / M). */
#define ALST_FLAG_REDUCE_SUM 4u

/* The dW sums are updated after EVERY tile instead of once per group of tiles, so the scratch holds
 * the bf16 dZ rows and the dense hidden rows of one tile only: workspace = O(tile * V) + O(V * H)
 * with the constant 1 (2 bytes per logit of one tile), the memory contract of Sequence Tiling to
 * the letter.  Without the flag the scratch holds a group of tiles (about 16384 rows: 8 tiles of
 * up to 2048 rows, 4 of 4096, 2 of 8192, 1 beyond), which saves the read-modify-write of the fp32
 * dW sums and the dW GEMM's start-up on all but the group's last tile.  Results agree to fp32
 * summation order. */
#define ALST_FLAG_TILE_SCRATCH 8u
/* alst_tiled_ce_workspace_bytes() / alst_tiled_ce_forward() / alst_tiled_ce_token_losses() only:
 * the workspace is sized for the forward pass alone (no dZ scratch, no dW sums); the entry points
 * that compute gradients return ALST_ERR_UNSUPPORTED for it. */
#define ALST_FLAG_FORWARD_ONLY 16u

/* Static, NUL-terminated description of a status value.  Host only. */
const char* alst_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch.  Host only. */
int alst_version(void);

/*
 * Bytes of device scratch the three compute entry points need for this problem, 0 if the
 * shape or the flags are invalid.  Pure host arithmetic, no device access.  The value is
 * independent of N except for about 12 * N bytes (per-row loss term, lse and dense-row index):
 * this is the memory contract of Sequence Tiling, peak = O(N * H) for the activations and their
 * gradients + O(tile * V) + O(V * H).  With Tp, Vp = tile and V rounded up to 256 the large terms are
 *   2 * Kg * (Vp + H)   bf16 dZ rows and dense hidden rows of the Kg rows in flight: Kg = Tp with
 *                       ALST_FLAG_TILE_SCRATCH, else Tp * clamp(16384 / Tp, 1, 8) (a group of tiles)
 *   4 * V * H           fp32 dW sums (absent for fp32 overwrite output, whose sums live in dW)
 *   2 * Vp * H          bf16 copy of W transposed, made once per call that computes gradients (the
 *                       dHidden product then reads both its operands along their rows)
 *   8 * (Vp / 128) * Tp   softmax partials of one tile
 * and with ALST_FLAG_FORWARD_ONLY only the last one and 2 * Tp * H remain.
 */
size_t alst_tiled_ce_workspace_bytes(int64_t N, int64_t H, int64_t V, int64_t tile, uint32_t flags);

/*
 * Forward only: mean cross-entropy of the tiled LM-head projection (one logits sweep, 2NHV flop).
 *   hidden  [N,H] bf16, W [V,H] bf16, labels [N] int32     inputs, not modified
 *   loss_out    [1] fp32    mean over non-ignored tokens
 *   lse_out     [N] fp32    per-row log-sum-exp of the tokens that take part, the only state
 *                           backward needs; 0 for ignored tokens (their rows are skipped: they
 *                           enter neither the loss nor a gradient); may be NULL
 *   n_valid_out [1] int64   number of non-ignored tokens; may be NULL
 */
int alst_tiled_ce_forward(const void* hidden, const void* W, const int32_t* labels,
                          int64_t N, int64_t H, int64_t V, int64_t tile, int32_t ignore_index,
                          float* loss_out, float* lse_out, int64_t* n_valid_out,
                          void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Backward only, from the lse a forward call produced (recomputes each tile's logits: 6NHV flop).
 *   lse       [N] fp32      from alst_tiled_ce_forward (entries of ignored tokens are not read)
 *   grad_loss host scalar   upstream gradient g of the loss (1.0f normally)
 *   dHidden   [N,H] bf16    overwritten, every row; rows of ignored tokens are exactly 0
 *   dW        [V,H] bf16 (fp32 with ALST_FLAG_DW_FP32); overwritten, or += with
 *             ALST_FLAG_DW_ACCUMULATE.  Accumulation over the tiles is always fp32.
 */
int alst_tiled_ce_backward(const void* hidden, const void* W, const int32_t* labels,
                           const float* lse,
                           int64_t N, int64_t H, int64_t V, int64_t tile, int32_t ignore_index,
                           float grad_loss, void* dHidden, void* dW,
                           void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Forward and backward of every tile in one sweep, as the paper's method does it (section
 * "Sequence Tiling for Reducing Activation Memory Footprint": forward and backward of a logits
 * shard are done together, shard by shard): 6NHV flop, each tile's logits are computed once.
 * Arguments as in the two calls above; lse_out and n_valid_out may be NULL.
 */
int alst_tiled_ce_forward_backward(const void* hidden, const void* W, const int32_t* labels,
                                   int64_t N, int64_t H, int64_t V, int64_t tile,
                                   int32_t ignore_index, float grad_loss,
                                   float* loss_out, float* lse_out, int64_t* n_valid_out,
                                   void* dHidden, void* dW,
                                   void* workspace, size_t workspace_bytes, uint32_t flags,
                                   void* stream);

/*
 * For callers that cannot allocate device memory and therefore cannot bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation
 * and same results, bit for bit, as alst_tiled_ce_forward_backward, with the workspace taken from
 * a buffer of ALST_NOALLOC_SCRATCH_BYTES that is part of the library's device code (every GPU the
 * library's kernels are loaded on holds one until the process ends).  The call allocates and
 * frees nothing, on the device or through any library.
 *   - A problem whose alst_tiled_ce_workspace_bytes(N, H, V, tile, flags) exceeds
 *     ALST_NOALLOC_SCRATCH_BYTES is refused with ALST_ERR_NOALLOC_LIMIT before anything is
 *     enqueued (ALST_FLAG_TILE_SCRATCH and ALST_FLAG_DW_FP32 lower the need; the LM-head
 *     workloads with V * H in the hundreds of millions do not fit: they need the caller's
 *     workspace for the fp32 dW sums alone).
 *   - device_status_out [1] int32, device, may be NULL: receives the status word the kernels
 *     leave (ALST_OK, ALST_ERR_LABEL_RANGE or ALST_ERR_NONFINITE), since the caller has no
 *     workspace to hand to alst_last_device_status.
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (two
 *     streams, two host threads) race and give wrong results; order them on one stream.  The
 *     buffer keeps the last call's contents; every call resets what it needs.
 *   - As for the other entry points, the first compute call on a device must be made outside a
 *     graph capture.
 * ALST_FLAG_FORWARD_ONLY is refused (ALST_ERR_UNSUPPORTED).
 */
#define ALST_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
int alst_tiled_ce_forward_backward_noalloc(const void* hidden, const void* W, const int32_t* labels,
                                           int64_t N, int64_t H, int64_t V, int64_t tile,
                                           int32_t ignore_index, float grad_loss,
                                           float* loss_out, float* lse_out, int64_t* n_valid_out,
                                           void* dHidden, void* dW, int32_t* device_status_out,
                                           uint32_t flags, void* stream);

/*
 * Synchronises `stream`, then reads and clears the device status word that the last call on this
 * workspace left: ALST_OK, ALST_ERR_LABEL_RANGE or ALST_ERR_NONFINITE (ALST_ERR_HIP if the copy
 * fails).  `workspace` must be one that a compute entry point has used.
 */
int alst_last_device_status(void* workspace, void* stream);

/*
 * The unreduced loss: token_loss_out[i] = lse[i] - z[i, label_i] for every non-ignored token and 0
 * for ignored ones, [N] fp32, as left in `workspace` by the last alst_tiled_ce_forward or
 * alst_tiled_ce_forward_backward call on it with the same N, H, V, tile and flags (the per-token
 * loss computations the paper's section "Sequence Tiling ..." lists among the operations without
 * cross-sequence dependency).  Enqueued on `stream` after that call.  workspace_bytes is checked
 * against alst_tiled_ce_workspace_bytes() of the same arguments (ALST_ERR_WORKSPACE).
 */
int alst_tiled_ce_token_losses(const void* workspace, size_t workspace_bytes, int64_t N, int64_t H,
                               int64_t V, int64_t tile, uint32_t flags, float* token_loss_out,
                               void* stream);

/*
 * Label utility for the boundary convention above (section "Loss Sharding in Hugging Face
 * Transformers"): shift_labels[i] = labels[i+1] for i < N-1, shift_labels[N-1] = ignore_index,
 * done on the whole sequence BEFORE it is cut along the sequence dimension, so no shard loses
 * its first label.  labels and shift_labels are device int32 [N] and must not overlap.
 */
int alst_shift_labels(const int32_t* labels, int32_t* shift_labels, int64_t N,
                      int32_t ignore_index, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ALST_H */
