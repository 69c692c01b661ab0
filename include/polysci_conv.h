/*
 * polysci_conv.h -- C ABI of the MI355X (gfx950) forward-convolution library.
 *
 * The library computes the forward 2-D convolution of the paper's Fig. 4 (Section 5,
 * "The 2-D Convolution code") on the blocked tensor layouts that figure's index
 * expressions define, as a grid of workgroups (the figure's outer loops) around a
 * batch-reduce GEMM microkernel on the matrix cores (the figure's "GEMM operation"),
 * plus the layout transforms into and out of the blocked layouts and the host-side
 * tile-selection model (the analogue of Section 4's working-set ranking).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or keeps them.  They must be 16-byte aligned and must not alias.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call
 *     only enqueues work on that stream and returns; there is no hidden synchronisation.
 *   - Return value: PS_OK (0) or a negative ps_status.  A call that fails validation
 *     launches nothing.  No C++ exception crosses this boundary.
 *   - Descriptors are plain structs passed by pointer; the library copies what it needs.
 *
 * Layouts (B = 16, Cb = ceil(C/16), Kb = K/16; es = 4 bytes for PS_F32, 2 for PS_BF16)
 *   activations, blocked : [N][Cb][H][W][16 c]              element size es
 *   filters, blocked     : [Kb][Cb][R][S][16 c][16 k]       PS_F32            (k fastest)
 *                          [Kb][Cb][R][S][2][16 k][8 c]     PS_BF16: block entry (c, k) sits at [c/8][k][c%8],
 *                                                           the reduction index packed for 16-bit MFMA operands
 *   outputs, blocked     : [N][Kb][P][Q][16 k]              always fp32
 *   plain tensors        : NCHW, KCRS, NKPQ, dense
 * Channel lanes c >= C of the blocked tensors hold +0.0.  K must be a multiple of 16.
 * Padding is logical: the blocked input is H x W, out-of-image taps contribute zero.
 * P = floor((H + 2*pad - R)/stride) + 1, Q likewise with W and S.
 */
#ifndef POLYSCI_CONV_H
#define POLYSCI_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PS_OK = 0,
    PS_EINVAL = -1,       /* null pointer, non-positive size, P or Q <= 0, misaligned pointer */
    PS_EUNSUPPORTED = -2, /* K % 16 != 0, unknown dtype, tensor too large for 32-bit element offsets,
                             tile not valid for this descriptor */
    PS_EHIP = -3,         /* the HIP runtime reported an error at launch */
    PS_ESCRATCH = -4      /* ps_conv2d_fwd_static: the tile needs more scratch than PS_STATIC_SCRATCH_BYTES */
} ps_status;

typedef enum { PS_F32 = 0, PS_BF16 = 1 } ps_dtype; /* element type of input and filter */

/* Problem sizes of one convolution: the loop bounds and strides of Fig. 4 (nImg, nIfm, ifh,
 * ifw, nOfm, kh, kw, STRIDE_H = STRIDE_W = stride) plus the symmetric zero padding that
 * Section 2 lists among the layer parameters. */
typedef struct {
    int32_t N, C, H, W, K, R, S, stride, pad;
    int32_t dtype; /* ps_dtype */
} ps_conv_desc;

/* One point of the outer-loop variant space (Section 4.2: tiling and interchange of the
 * loops around the microkernel, with varied tile sizes), in GPU terms:
 *   kt      output channels per workgroup tile (32, 64, 128 or 256)
 *   mt      output pixels per workgroup tile, counted in the flattened (n, p, q) order (32 ... 256 in steps of 32
 *           on 32x32 MFMA tiles; 48, 96 or 176 on 16x16 MFMA tiles, fp32 only: kt = 64, or kt = 256 for the 1x1
 *           kernels that keep the pixels in LDS and walk over four 64-channel tiles)
 *   ring    batch-reduce elements (c-block, r, s) resident in the LDS ring, i.e. how far ahead of the
 *           matrix cores the global loads run (2, 4 or 8)
 *   c_split workgroups that share one output tile, each reducing a contiguous slice of the
 *           (c-block, r, s) range; > 1 accumulates with atomic adds into a cleared output
 *   raster  launch order of tiles: 0 = output-channel tiles fastest, 1 = pixel tiles fastest
 */
typedef struct {
    int32_t kt, mt, ring, c_split, raster;
} ps_tile;

/* Output size of `d`.  PS_EINVAL if the descriptor is invalid. */
int ps_out_dims(const ps_conv_desc *d, int32_t *P, int32_t *Q);

/* Bytes of the blocked tensors of `d` (0 if the descriptor is invalid). */
size_t ps_blocked_in_bytes(const ps_conv_desc *d);  /* N*Cb*H*W*16*es        */
size_t ps_blocked_wt_bytes(const ps_conv_desc *d);  /* Kb*Cb*R*S*256*es      */
size_t ps_blocked_out_bytes(const ps_conv_desc *d); /* N*Kb*P*Q*16*4         */

/* ---- layout transforms (bit-exact permutations; Fig. 4 index expressions) -------------- */
/* NCHW (N*C*H*W elements of size es) -> blocked activations; pad lanes written as +0.0. */
int ps_nchw_to_blocked(const ps_conv_desc *d, const void *nchw, void *blk, void *stream);
/* blocked activations -> NCHW (pad lanes dropped). */
int ps_blocked_to_nchw(const ps_conv_desc *d, const void *blk, void *nchw, void *stream);
/* KCRS -> blocked filters; pad c lanes written as +0.0. */
int ps_kcrs_to_blocked(const ps_conv_desc *d, const void *kcrs, void *wblk, void *stream);
/* blocked filters -> KCRS. */
int ps_blocked_to_kcrs(const ps_conv_desc *d, const void *wblk, void *kcrs, void *stream);
/* blocked fp32 output [N][Kb][P][Q][16] -> NKPQ fp32. */
int ps_blocked_to_nkpq(const ps_conv_desc *d, const void *oblk, void *nkpq, void *stream);

/* ---- forward convolution ------------------------------------------------------------- */
/* out_blk = conv(in_blk, wt_blk) on blocked tensors; out_blk is overwritten (the "+=" of
 * Fig. 4 applied to a cleared output).  The workgroup tile is the tile model's pick (ps_tile_pick: ranked once per
 * descriptor, then served from the per-process table). */
int ps_conv2d_fwd(const ps_conv_desc *d, const void *in_blk, const void *wt_blk, void *out_blk,
                  void *stream);
/* Same with an explicit tile (autotune sweeps).  PS_EUNSUPPORTED if ps_tile_valid fails. */
int ps_conv2d_fwd_tile(const ps_conv_desc *d, const ps_tile *t, const void *in_blk,
                       const void *wt_blk, void *out_blk, void *stream);

/* Workspace variant for split reductions (c_split > 1): each split stores its partial tile into its own
 * plane of `workspace` with plain stores and a second kernel adds the planes into out_blk; nothing is
 * cleared and no atomics are used, so the result does not depend on arrival order.  `workspace` is a device
 * buffer of at least ps_workspace_bytes(d, t) bytes, owned by the caller, 16-byte aligned, scratch (contents
 * undefined afterwards); it may be NULL when the tile needs none.  t == NULL runs ps_tile_select_ws's pick
 * for the given workspace size.  PS_EINVAL if the workspace is too small for the tile. */
size_t ps_workspace_bytes(const ps_conv_desc *d, const ps_tile *t); /* c_split * N*K*P*Q*4, 0 if c_split == 1 */
int ps_conv2d_fwd_ws(const ps_conv_desc *d, const ps_tile *t, const void *in_blk, const void *wt_blk,
                     void *out_blk, void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory and have no workspace to lend (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): ps_conv2d_fwd_ws with the workspace replaced by an array the
 * library holds in static device memory, PS_STATIC_SCRATCH_BYTES (64 MiB) per GPU, there until the process ends.
 * The call allocates and frees nothing on the device and calls no allocating runtime routine; the caller passes only
 * inputs and outputs.  t == NULL runs the pick among the tiles whose partial planes fit the array (ps_tile_pick with
 * workspace_bytes = PS_STATIC_SCRATCH_BYTES); an explicit tile whose planes need more (ps_workspace_bytes) returns
 * PS_ESCRATCH and launches nothing.  Results are those of ps_conv2d_fwd_ws with the same tile, bit for bit.
 * The array keeps the last call's contents; nothing in it has to start at zero (every plane element that is read
 * was stored by the same call), so nothing is cleared.  All calls on one GPU share that GPU's array: calls that can
 * overlap in time on one GPU (different streams, different threads) race on it and must be ordered by the caller.
 * The array's device address is looked up on the first call on each device (one symbol query, kept afterwards);
 * make that first call outside stream capture. */
#define PS_STATIC_SCRATCH_BYTES (64u << 20)
int ps_conv2d_fwd_static(const ps_conv_desc *d, const ps_tile *t, const void *in_blk, const void *wt_blk,
                         void *out_blk, void *stream);

/* Convolution with the work of the following layers of an inference pipeline fused into the store of the output
 * tile (Section 5 evaluates the convolutions of such pipelines; what follows each one there is a bias, an activation
 * and the next convolution).  y = conv(in, wt) as above, then in this order:
 *   bias      != NULL: y[n][k][p][q] += bias[k]   (device pointer to K fp32 values, 16-byte aligned)
 *   relu      != 0   : y = max(y, 0)
 *   out_dtype        : PS_F32 stores y as ps_conv2d_fwd does; PS_BF16 rounds y to bf16 (nearest, ties to even) and
 *                      stores [N][Kb][P][Q][16 k] with 2-byte elements (N*K*P*Q*2 bytes).
 * Either way out_blk has exactly the blocked activation layout of a next layer with C = K, H = P, W = Q of that
 * element type, so layers chain with no transform in between.  Tile and workspace as for ps_conv2d_fwd_ws; a tile
 * with c_split > 1 needs its workspace (PS_EINVAL without), because the epilogue is applied where the sum is
 * complete. */
typedef struct {
    const void *bias;
    int32_t relu;
    int32_t out_dtype; /* ps_dtype */
} ps_epilogue;
int ps_conv2d_fwd_fused(const ps_conv_desc *d, const ps_tile *t, const ps_epilogue *e, const void *in_blk,
                        const void *wt_blk, void *out_blk, void *workspace, size_t workspace_bytes, void *stream);

/* ---- outer-loop variant space and its ranking (Section 4.2, Algorithm 2, Eq. 1) ------- */
/* Number of candidate tiles the enumerator emits for `d` (negative ps_status on error). */
int ps_tile_count(const ps_conv_desc *d);
/* The idx-th candidate, 0 <= idx < ps_tile_count(d). */
int ps_tile_get(const ps_conv_desc *d, int idx, ps_tile *t);
/* PS_OK if `t` can run `d` (a compiled kernel shape exists and the split divides evenly). */
int ps_tile_valid(const ps_conv_desc *d, const ps_tile *t);
/* Modelled execution time of `t` on `d` in microseconds; negative if invalid.  ps_tile_cost_us prices a
 * split reduction as ps_conv2d_fwd_tile runs it (clear + atomics), ps_tile_cost_ws_us as ps_conv2d_fwd_ws
 * runs it (partial planes + reduction pass). */
double ps_tile_cost_us(const ps_conv_desc *d, const ps_tile *t);
double ps_tile_cost_ws_us(const ps_conv_desc *d, const ps_tile *t);
/* The candidate with the lowest modelled time (k = 1 of the paper's top-k pick). */
int ps_tile_select(const ps_conv_desc *d, ps_tile *best, double *modelled_us);
/* Same for ps_conv2d_fwd_ws: only candidates whose workspace fits in `workspace_bytes` compete. */
int ps_tile_select_ws(const ps_conv_desc *d, size_t workspace_bytes, ps_tile *best, double *modelled_us);
/* The paper's protocol in full (Section 4.2: rank the n variants, run the top k on the target, keep the fastest):
 * writes the k candidates with the lowest modelled time, best first, to tiles[0..] (host memory, room for k entries;
 * modelled_us may be NULL, else room for k values) under the rules of ps_tile_select_ws, and returns how many were
 * written (fewer than k if the layer has fewer candidates), or a negative ps_status.  tiles[0] is the tile
 * ps_tile_select_ws returns.  Timing the k tiles is the caller's part (paper_2002_02145_amd.autotune.run_top_k). */
int ps_tile_rank_ws(const ps_conv_desc *d, size_t workspace_bytes, int k, ps_tile *tiles, double *modelled_us);

/* Environment (read when a descriptor is first ranked by a convolution call or ps_tile_pick, then cached with the pick):
 *   PS_FORCE_TILE="kt,mt,ring,c_split,raster"  use this tile wherever it is valid (and its workspace fits) instead of
 *                                              the model's pick: a way to pin or A/B a tile without changing callers;
 *   PS_DUMP_RANKING=k                          print the k best candidates and their modelled times to stderr. */
/* The tile the convolution calls run when none is passed: ps_conv2d_fwd (with_workspace = 0, ranking of
 * ps_tile_select) or ps_conv2d_fwd_ws / ps_conv2d_fwd_fused with t == NULL (with_workspace != 0, ranking of
 * ps_tile_select_ws for `workspace_bytes`).  The ranking of Section 4.2 depends on the descriptor alone, so the
 * library computes it on first use and keeps it, together with the prepared launch of every (descriptor, tile) pair
 * it has run, in a per-process table: entries are immutable once published, lookups are thread-safe, steady-state
 * cost is a hash lookup instead of pricing every candidate.  What a workspace size decides is how many partial planes
 * fit (at most 16), so sizes with the same count share an entry.  The table holds at most 16384 entries of each
 * kind; beyond that, results are computed per call as ps_tile_select does.  ps_tile_cache_entries reports how many
 * entries (picks plus prepared launches) the process holds. */
int ps_tile_pick(const ps_conv_desc *d, int with_workspace, size_t workspace_bytes, ps_tile *t);
size_t ps_tile_cache_entries(void);

/* Section 4.2's protocol carried out by the library itself: the n variants are ranked by the model, the best k (at most
 * 16) are run on the target, the fastest is kept.  The candidates are those of ps_tile_rank_ws for `workspace_bytes`;
 * each is launched on the caller's blocked tensors a few times and timed with events on `stream` (out_blk ends up
 * holding the convolution's result; workspace as for ps_conv2d_fwd_ws, NULL if none is lent).  The winner replaces the
 * descriptor's entry in the per-process table, so later convolution calls with t == NULL and a workspace of the same
 * class run it (and ps_conv2d_fwd too, if the winner is not a split tile).  This is the one convolution-side call that
 * waits for its stream: use it at set-up, not in the serving path.  Returns the number of candidates timed, or a
 * negative ps_status; *best and *best_us (either may be NULL) receive the winner and its microseconds per launch. */
int ps_tile_autotune(const ps_conv_desc *d, int k, const void *in_blk, const void *wt_blk, void *out_blk, void *workspace,
                     size_t workspace_bytes, void *stream, ps_tile *best, double *best_us);

/* Which inner loop the library runs for tile `t` on `d` (for reports and tests): the loop with a runtime filter size,
 * the loops with a 1x1, 3x3 or 5x5 filter baked in, the loops for 3x3, 5x5, 7x7 and 11x11 filters over at most 3 (fp32; 7x7:
 * 4) or 8 (16-bit) input channels that pack four (two) taps into one batch element, the 16-bit 3x3 loop that stages the input patch once per c-block, or the fp32 1x1 loop that keeps a
 * tile's pixels with all 64 input channels in LDS and walks over four 64-channel output tiles (tile kt = 256).
 * Negative ps_status if the tile is not valid for the descriptor. */
typedef enum {
    PS_KERNEL_GENERAL = 0,
    PS_KERNEL_1X1 = 1,
    PS_KERNEL_STATIONARY_1X1 = 2,
    PS_KERNEL_3X3 = 3,
    PS_KERNEL_5X5 = 5,
    PS_KERNEL_PACKED_TAPS = 7,
    PS_KERNEL_PATCH_3X3 = 9
} ps_kernel_variant;
int ps_tile_kernel(const ps_conv_desc *d, const ps_tile *t);

/* Measurement aid for reports (no part of the method): launches a loop of `iters` x 32 independent MFMAs per wave
 * of the given element type (fp32: 16x16x4, bf16: 32x32x16) on 16 waves per compute unit, with no operand traffic,
 * and writes the FLOP it performs to *flop (host pointer, may be NULL).  Timed by the caller with events on `stream`,
 * it gives the rate the matrix cores of this device sustain, to put next to the published peak.  `sink` is a device
 * buffer of at least 1 KB that the kernel never actually writes. */
int ps_probe_mfma(int dtype, int iters, void *sink, double *flop, void *stream);

const char *ps_strerror(int status);
/* The HIP runtime's description of the last PS_EHIP this thread received ("" if none); static storage. */
const char *ps_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* POLYSCI_CONV_H */
